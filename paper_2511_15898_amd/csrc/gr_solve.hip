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
// with power series in z truncated at degree n and the trapezoid rule in log t.  The product is taken
// through its logarithm: log(1 + x (e^u - 1)) = sum_k kappa_k(x) u^k / k! with the cumulants of a
// Bernoulli(x) variable, and only k <= n can reach the z^n coefficient, so n cumulant sums per
// quadrature node describe all tokens exactly; the series exponential is taken once per node.
#include "gr_internal.h"
#include "gr_verify_row.h"

namespace gr {

// The workgroup's LDS (dynamic: its size is that of Lds<D>), named at file scope so that functions that are not
// inlined address it as LDS and not through generic pointers.
extern __shared__ __align__(16) unsigned char gr_lds_raw[];

namespace {

// Optional cycle accounting (builds with -DGR_PHASE_CLOCKS only): thread 0 adds the shader-clock cycles since
// its previous mark to one of 24 slots; the totals per row are written to RowInfo::clk.
#ifdef GR_PHASE_CLOCKS
#define GR_CLK(L, slot) do { if (threadIdx.x == 0) { const long long now_ = clock64(); (L).clk[slot] += now_ - (L).clk_last; (L).clk_last = now_; } } while (0)
#else
#define GR_CLK(L, slot) do {} while (0)
#endif

constexpr int KS = kMaxSupport;
// Threads of the solve workgroup: eight waves (two per SIMD, 256 registers each) up to 8 drafts, so that one
// wave's dependent float64 chains and LDS waits are filled by the other; four waves (one per SIMD, all 512
// registers) for the longer series of 9 to 16 drafts.
#ifndef GR_THREADS_UP_TO_8
#define GR_THREADS_UP_TO_8 512
#endif
template <int D> constexpr int kThreadsOf = D > 8 ? 256 : GR_THREADS_UP_TO_8;
constexpr double kQuadStep = 0.45;   // trapezoid step in log t (discretisation error ~1e-9 relative)
constexpr double kQuadLo = 1e-4;     // t_lo * (slack + sum w): the part below t_lo is added in closed form
constexpr double kQuadHi = 25.0;     // t_hi * (slowest decay rate)
constexpr double kStretch = 4.0;     // first cap on the per-coordinate stretch of the fixed-point step
constexpr int kStall = 3;            // iterations without a better point before the cap is halved
constexpr double kOddsFrom = 0.9, kOddsTo = 0.999;    // targets within these shares of Pr[token drawn] ...
constexpr double kOddsFirst = 0.5;                    // ... that start further than this from their routed mass (in log) step on the log odds ...
constexpr double kOddsUntil = 1e-6;                   // ... while the stopping measure is above this
constexpr int kMixBudget = 60;       // the mixed fixed-point iteration gets kMixBudget + m evaluations before Newton takes over
constexpr int kCols = kHist - 1;                       // Anderson columns
constexpr int kMaxHeavy = 3;         // tokens that keep their exact factor (only with more than 8 drafts)
constexpr double kHeavyShare = 0.3;  // ... those above this share of the program's draw mass

// Operands of one token / one quadrature node, packed so that they are a few 16-byte LDS reads.
template <int D> struct alignas(16) TokRec { double aw; double e[D]; double pad; };     // weight; e[k-1] = q^k / k! (0 for k > n)
template <int D> struct alignas(16) NodeRec { double t, qw; double Tr[D]; };            // abscissa, quadrature weight; Tr[k-1] = T_{n-k}

// The quadrature grid of one evaluation: nodes t_lo e^{step j}, j = 0..N-1, and the closed-form sums over the
// nodes below t_lo (x = 1 there) of the integral of 1 (tail) and of t (tail2).
struct Grid { double t_lo, step, tail, tail2; int N; };

// D: the series degree of the kernel (>= n).
template <int D>
struct Lds {
    static constexpr int kST = kThreadsOf<D>;
    static constexpr int kSW = kST / 64;
    static constexpr int kNPW = 64 / kSW;   // quadrature nodes a wave owns within a chunk of 64
    // support, in ratio order
    int tok[KS]; int blk[KS]; int inT[KS]; int ordq[KS]; int apos[kMaxT];
    int flag[KS + 2]; int blo[KS + 2];
    double qn[KS]; double pn[KS]; double rho[KS]; double tgt[KS]; double wgt[KS];
    double Q[KS + 1]; double F[KS + 2];
    // one convex program (tokens by decreasing q)
    double aq[kMaxT]; double at[kMaxT]; double aal[kMaxT]; double aR[kMaxT];
    double aS[kMaxT]; double ag[kMaxT];   // with aR: what one evaluation hands to the mixing step (see solve_program)
    int aodds[kMaxT];                     // tokens that step on their log odds (chosen at a program's first evaluation)
    double aR0, alc;                      // ... the slack mass and, with slack, log(slack mass / its target)
    double ared[2][3];                    // ... and the first two waves' sum of R, max and min of log(target / R)
    double apd[kMaxT];              // Pr[token drawn within the program] = atot^n - (atot - q)^n
    double aw[kMaxT]; double af[kMaxT]; int adeg[kMaxT];   // staging of the HBM-path programs kernel
    // Newton fallback (its Jacobian lives in a per-row HBM scratch)
    double nR[kMaxT]; double nstep[kMaxT]; double nsave[kMaxT]; int nused[kMaxT]; int ncolof[kMaxT];
    // scans and counters of the prologue (dead once the first program starts) share their bytes with the
    // evaluator's records and per-wave partial sums
    union {
        struct {
            int cnt0[KS + 2]; int cnt1[KS + 2]; int ids[KS]; int byq[KS];
            double qd[KS]; double accb[KS];
            double dlt[KS]; double dval[KS];   // rows given as logits: draft minus target logit, draft logit
            double P[KS + 1]; double S[KS + 1]; double G0[KS + 2]; double G1[KS + 2];
        };
        struct {
            double rpart[kSW][kMaxT];   // per wave: sum over its nodes of the integrand of each token
            double spart[kSW][kMaxT];   // the same weighted by t
            NodeRec<D> nrec[kSW][kNPW];
            TokRec<D> trec[kMaxT + 4];  // active tokens; every record beyond the last has aw = 1e300 (x = 0), e = 0
        };
    };
    double Ha[kHist][kMaxT]; double Hf[kHist][kMaxT]; double aBest[kMaxT]; double fBest[kMaxT]; double rBest[kMaxT];
    double pm[kHist][kHist];        // inner products of the stored residual vectors of the mixing, by history slot
    Grid ctl_grid; int ctl_go, ctl_result, ctl_bestok;   // handed from the mixing wave to all waves
    double e2tab[32];               // 2^(-j/32)
    int nheavy;                     // leading tokens that keep their exact factor
    int nfull;                      // leading tokens (the heavy ones included) that need all D cumulants; the rest need four
    double work;                    // sum over evaluator calls of nodes x active tokens (thread 0 only)
#ifdef GR_PHASE_CLOCKS
    long long clk[24]; long long clk_last; double errlog[24];
#endif
    double red[2][kSW][8]; double redn[kSW]; double r0part[kSW]; int pick[4]; int count; int hist[256];
    unsigned long long keys[kSelCap];   // unsorted candidates (select merge)
};

// ---- workgroup reductions with one barrier: the waves' partial results alternate between two LDS
// strips (`par`), so the strip of the reduction before the previous one is free again.
enum { kOpSum = 0, kOpMax = 1, kOpMin = 2 };
__device__ __forceinline__ double combine(double a, double b, int op) {
    return op == kOpSum ? a + b : (op == kOpMax ? fmax(a, b) : fmin(a, b));
}
// Several reductions over the lanes of one wave at once (their butterfly steps interleave): every lane ends with
// the results.  All 64 lanes must be active.
template <int NV>
__device__ __forceinline__ void wave_reduce_many(double (&v)[NV], const int (&op)[NV]) {
#pragma unroll
    for (int j = 0; j < NV; ++j) v[j] = combine(v[j], dpp_move<kDppXor1>(v[j]), op[j]);
#pragma unroll
    for (int j = 0; j < NV; ++j) v[j] = combine(v[j], dpp_move<kDppXor2>(v[j]), op[j]);
#pragma unroll
    for (int j = 0; j < NV; ++j) v[j] = combine(v[j], dpp_move<kDppHalfMirror>(v[j]), op[j]);
#pragma unroll
    for (int j = 0; j < NV; ++j) v[j] = combine(v[j], dpp_move<kDppMirror>(v[j]), op[j]);
#pragma unroll
    for (int j = 0; j < NV; ++j)
        v[j] = combine(combine(read_lane(v[j], 0), read_lane(v[j], 16), op[j]), combine(read_lane(v[j], 32), read_lane(v[j], 48), op[j]), op[j]);
}

// v[j] holds this wave's partial result of operation op[j]; on return it holds the workgroup's.  After the
// barrier lane l reads the partial of wave l mod NW (one LDS instruction per value and wave, not NW), and a
// butterfly over NW neighbouring lanes combines them: every lane ends with the same bits.
template <int NV, class LdsT>
__device__ __forceinline__ void wg_reduce(LdsT& L, int& par, double (&v)[NV], const int (&op)[NV]) {
    constexpr int NW = LdsT::kSW;
    static_assert(NW == 4 || NW == 8, "the butterfly below covers four or eight waves");
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    if (lane == 0) {
#pragma unroll
        for (int j = 0; j < NV; ++j) L.red[par][wv][j] = v[j];
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        double r = L.red[par][lane & (NW - 1)][j];
        r = combine(r, dpp_move<kDppXor1>(r), op[j]);
        r = combine(r, dpp_move<kDppXor2>(r), op[j]);
        if (NW == 8) r = combine(r, dpp_move<kDppHalfMirror>(r), op[j]);
        v[j] = r;
    }
    par ^= 1;
}
template <class LdsT> __device__ __forceinline__ double wg_sum(LdsT& L, int& par, double v) {
    double a[1] = {wave_sum(v)};
    wg_reduce<1>(L, par, a, {kOpSum});
    return a[0];
}
template <class LdsT> __device__ __forceinline__ double wg_max(LdsT& L, int& par, double v) {
    double a[1] = {wave_max(v)};
    wg_reduce<1>(L, par, a, {kOpMax});
    return a[0];
}

// 1/x from the hardware estimate and two Newton steps (about 1e-16 relative; x = 0, infinite or NaN gives NaN or 0).
__device__ __forceinline__ double fast_rcp(double x) {
    double r = __builtin_amdgcn_rcp(x);
    r = r * fma(-x, r, 2.0);
    r = r * fma(-x, r, 2.0);
    return r;
}

// e^x for |x| <= 1000 (clamped beyond) with the table of exp_neg: x = -(k ln2/32 + r), k of either sign.
__device__ __forceinline__ double exp_signed(double x, const double* tab) {
    const double y = fmax(fmin(-x, 1000.0), -1000.0);
    const double kf = rint(y * 46.166241308446828);
    const int ki = static_cast<int>(kf);
    const double tv = tab[ki & 31];                            // k = 32 (k >> 5) + (k & 31), also for negative k
    double r = fma(kf, -(6.93147180369123816490e-01 / 32.0), y);
    r = -fma(kf, -(1.90821492927058770002e-10 / 32.0), r);
    double p = 8.33333333333333333333e-03;
    p = fma(p, r, 4.16666666666666666667e-02);
    p = fma(p, r, 1.66666666666666666667e-01);
    p = fma(p, r, 0.5);
    p = fma(p, r, 1.0);
    p = fma(p, r, 1.0);
    return ldexp(p * tv, -(ki >> 5));
}

// log(x) to about 1e-16 relative for positive normal x: x = 2^e m with m in [sqrt(1/2), sqrt(2)),
// log m = 2 atanh(s) = 2 s (1 + s^2/3 + s^4/5 + ...), s = (m - 1) / (m + 1), |s| <= 0.172 (eleven terms).
// Anything else (zero, negative, denormal, infinite, NaN) goes to the library routine.
__device__ __forceinline__ double fast_log(double x) {
    if (!(x >= 2.3e-308 && x <= 1.7e308)) return log(x);
    int e;
    double m = frexp(x, &e);                                   // m in [1/2, 1)
    if (m < 0.70710678118654752) { m *= 2.0; e -= 1; }
    const double s = (m - 1.0) * fast_rcp(m + 1.0), z = s * s;
    double p = 1.0 / 21.0;
    p = fma(p, z, 1.0 / 19.0); p = fma(p, z, 1.0 / 17.0); p = fma(p, z, 1.0 / 15.0); p = fma(p, z, 1.0 / 13.0);
    p = fma(p, z, 1.0 / 11.0); p = fma(p, z, 1.0 / 9.0); p = fma(p, z, 1.0 / 7.0); p = fma(p, z, 1.0 / 5.0);
    p = fma(p, z, 1.0 / 3.0); p = fma(p, z, 1.0);
    const double ed = static_cast<double>(e);
    return fma(ed, 6.93147180369123816490e-01, fma(2.0 * s, p, ed * 1.90821492927058770002e-10));
}

// Cumulants of a Bernoulli(x) variable: kappa_1 = x, kappa_{k+1} = v g_k with v = x (1 - x),
// g_k = d kappa_k / dx = a_k(v) for odd k, s a_k(v) for even k, s = 1 - 2x (from kappa_{k+1} = x (1 - x) kappa_k').
// Row k: the coefficients of a_k in rising powers of v.
__device__ constexpr double kCumA[17][8] = {
    {0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0},
    {1.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0},
    {1.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0},
    {1.0, -6.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0},
    {1.0, -12.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0},
    {1.0, -30.0, 120.0, 0.0, 0.0, 0.0, 0.0, 0.0},
    {1.0, -60.0, 360.0, 0.0, 0.0, 0.0, 0.0, 0.0},
    {1.0, -126.0, 1680.0, -5040.0, 0.0, 0.0, 0.0, 0.0},
    {1.0, -252.0, 5040.0, -20160.0, 0.0, 0.0, 0.0, 0.0},
    {1.0, -510.0, 17640.0, -151200.0, 362880.0, 0.0, 0.0, 0.0},
    {1.0, -1020.0, 52920.0, -604800.0, 1814400.0, 0.0, 0.0, 0.0},
    {1.0, -2046.0, 168960.0, -3160080.0, 19958400.0, -39916800.0, 0.0, 0.0},
    {1.0, -4092.0, 506880.0, -12640320.0, 99792000.0, -239500800.0, 0.0, 0.0},
    {1.0, -8190.0, 1561560.0, -57657600.0, 726485760.0, -3632428800.0, 6227020800.0, 0.0},
    {1.0, -16380.0, 4684680.0, -230630400.0, 3632428800.0, -21794572800.0, 43589145600.0, 0.0},
    {1.0, -32766.0, 14217840.0, -988107120.0, 22313491200.0, -210680870400.0, 871782912000.0, -1307674368000.0},
    {1.0, -65532.0, 42653520.0, -3952428480.0, 111567456000.0, -1264085222400.0, 6102480384000.0, -10461394944000.0},
};

// g[k-1] = g_k(x) for k = 1..C.
template <int K, int C>
__device__ __forceinline__ void cum_g_from(double v, double s, double (&g)[C]) {
    if constexpr (K <= C) {
        constexpr int deg = (K - 1) / 2;
        double r = kCumA[K][deg];
#pragma unroll
        for (int j = deg - 1; j >= 0; --j) r = fma(r, v, kCumA[K][j]);
        g[K - 1] = (K % 2 == 0) ? r * s : r;
        cum_g_from<K + 1, C>(v, s, g);
    }
}

// A(z) <- A(z) * (1 + x (e^{zq} - 1)), e[a-1] = q^a / a!.
template <int D>
__device__ __forceinline__ void mul_factor(double (&A)[D + 1], double x, const double (&e)[D]) {
#pragma unroll
    for (int d = D; d >= 1; --d) {
        double acc = 0.0;
#pragma unroll
        for (int a = 1; a <= d; ++a) acc = fma(e[a - 1], A[d - a], acc);
        A[d] = fma(x, acc, A[d]);
    }
}

// [z^n] of  (e^{zq} - 1) * T(z) / (1 + x (e^{zq} - 1)): the leave-one-out coefficient of a token that
// keeps its exact factor, by series division (the quotient is only needed below degree n).
template <int D>
__device__ __forceinline__ double loo_coeff(const double (&T)[D + 1], double x, const double (&e)[D], int n) {
    double Bq[D + 1];
    Bq[0] = T[0];
    double cn = 0.0;
#pragma unroll
    for (int d = 1; d <= D; ++d) {
        double conv = 0.0;
#pragma unroll
        for (int a = 1; a <= d; ++a) conv = fma(e[a - 1], Bq[d - a], conv);
        Bq[d] = fma(-x, conv, T[d]);
        if (d == n) cn = conv;
    }
    return cn;
}

// rec.Tr[k-1] = T_{NN-k} (0 below degree 0); returns T_NN.
template <int D, int NN>
__device__ __forceinline__ double pick_series(NodeRec<D>& rec, const double (&T)[D + 1], int n) {
    if constexpr (NN >= 1) {
        if (n == NN) {
#pragma unroll
            for (int k = 1; k <= D; ++k) rec.Tr[k - 1] = (NN - k >= 0) ? T[(NN - k >= 0) ? NN - k : 0] : 0.0;
            return T[NN];
        }
        return pick_series<D, NN - 1>(rec, T, n);
    } else {
        return 0.0;
    }
}

// Phase 1, one token at one node: its cumulant terms into the node's sums, K[k-1] += kappa_k(x) q^k / k!
// for k <= C (C = D: exact; C = 4 for a token so small that its higher terms cannot reach the z^n
// coefficient within 1e-11).
template <int D, int C>
__device__ __forceinline__ void phase1_token(double (&K)[D], const TokRec<D>& r, double x) {
    const double v = fma(-x, x, x), s = fma(-2.0, x, 1.0);
    K[0] = fma(x, r.e[0], K[0]);
    if constexpr (C >= 2) {
        double g[C - 1];
        cum_g_from<1, C - 1>(v, s, g);
#pragma unroll
        for (int k = 2; k <= C; ++k) K[k - 1] = fma(v * g[k - 2], r.e[k - 1], K[k - 1]);
    }
}

// Tokens first + tsub, first + tsub + NS, ... below `last` at this lane's node, two records in flight.
template <int D, int C, int NS>
__device__ __forceinline__ void phase1_range(double (&K)[D], const TokRec<D>* trec, int first, int last, int pad, int tsub,
                                             double t, const double* tab) {
    if (first >= last) return;
    const int i0 = first + tsub;
    TokRec<D> cur = trec[i0 < last ? i0 : pad];
    for (int b = first; b < last; b += 2 * NS) {           // uniform trip count; the pad record has x = 0
        const int i1 = b + tsub + NS, i2 = b + tsub + 2 * NS;
        const TokRec<D> nxt = trec[i1 < last ? i1 : pad];
        double x0, x1;
        exp_neg2(t * cur.aw, t * nxt.aw, tab, x0, x1);
        phase1_token<D, C>(K, cur, x0);
        cur = trec[i2 < last ? i2 : pad];
        phase1_token<D, C>(K, nxt, x1);
    }
}

// Phase 3, one token at one node: (e^u - 1) / (1 + x (e^u - 1)) = sum_k g_k(x) u^k / k!, so the
// leave-one-out coefficient is sum_{k <= C} g_k(x) (q^k / k!) T_{n-k}.
template <int D, int C>
__device__ __forceinline__ void phase3_pair(const NodeRec<D>& c, const double (&e)[D], double x, double& acc, double& at) {
    const double v = fma(-x, x, x), s = fma(-2.0, x, 1.0);
    double g[C];
    cum_g_from<1, C>(v, s, g);
    double cn = e[0] * c.Tr[0];
#pragma unroll
    for (int k = 2; k <= C; ++k) cn = fma(e[k - 1] * g[k - 1], c.Tr[k - 1], cn);
    const double term = c.qw * x * cn;
    acc += term;
    at = fma(term, c.t, at);
}

// Tokens [first, last) against the npw nodes of this wave: lane = (token slot, node subset), the split that
// needs the fewest rounds; the sums go to this wave's rpart / spart.
template <int D, int C, class LdsT>
__device__ __forceinline__ void phase3_range(LdsT& L, int first, int last, int pad, int npw, int wv, int lane) {
    constexpr int NPW = LdsT::kNPW;
    const int cnt = last - first;
    if (cnt <= 0 || npw <= 0) return;
    // cost of a split in units of one (token, node) pair: per group of tokens the rounds over the node
    // subsets, one unit for loading the token and storing its sums, one per level of the butterfly
    int ts_log = 6, best = ((cnt + 63) >> 6) * (npw + 1);
#pragma unroll
    for (int tl = 5; tl >= 3; --tl) {
        const int nsub_ = 64 >> tl;
        if (nsub_ > NPW) break;
        const int c = ((cnt + (1 << tl) - 1) >> tl) * ((npw + nsub_ - 1) / nsub_ + 1 + (6 - tl));
        if (c < best) { best = c; ts_log = tl; }
    }
    const int TS = 1 << ts_log, nsub = 64 >> ts_log;
    const int tslot = lane & (TS - 1), ns = lane >> ts_log;
    const int rounds = (npw + nsub - 1) / nsub;
    for (int g0 = first; g0 < last; g0 += TS) {
        const int tok = g0 + tslot;
        const TokRec<D> tr = L.trec[tok < last ? tok : pad];
        double acc = 0.0, at = 0.0;
        NodeRec<D> cur = L.nrec[wv][ns];
        for (int r = 0; r < rounds; r += 2) {
            const int j1 = ns + (r + 1) * nsub, j2 = ns + (r + 2) * nsub;
            const NodeRec<D> nxt = L.nrec[wv][j1 < NPW ? j1 : ns];
            double x0, x1;
            exp_neg2(cur.t * tr.aw, nxt.t * tr.aw, L.e2tab, x0, x1);
            phase3_pair<D, C>(cur, tr.e, x0, acc, at);
            cur = L.nrec[wv][j2 < NPW ? j2 : ns];
            if (r + 1 < rounds) phase3_pair<D, C>(nxt, tr.e, x1, acc, at);
        }
        if (ts_log <= 5) { acc += __shfl_xor(acc, 32); at += __shfl_xor(at, 32); }
        if (ts_log <= 4) { acc += __shfl_xor(acc, 16); at += __shfl_xor(at, 16); }
        if (ts_log <= 3) { acc += __shfl_xor(acc, 8); at += __shfl_xor(at, 8); }
        if (ns == 0 && tok < last) { L.rpart[wv][tok] += acc; L.spart[wv][tok] += at; }
    }
}

// The evaluator for up to eight drafts takes phase 3 in two parts: the first CL terms, which every token needs, and
// the terms CL + 1 .. D of a token that needs them all.
// Phase 3: the sum of phase3_pair by Horner's rule in q = e[0], with Tp[k-1] = T_{n-k} / k!, so that only q is read:
//   cn = q (Tp_1 + q (g_2 Tp_2 + ... + q (g_CL Tp_CL + q top))),  top = g_{CL+1} Tp_{CL+1} + q (... + q g_D Tp_D)
// for a token that needs all terms, top = 0 otherwise.
template <int D, int CL>
__device__ __forceinline__ double loo_top(const double (&Tp)[D], double q, double v, double s) {
    if constexpr (D > CL) {
        double g[D];
        cum_g_from<CL + 1, D>(v, s, g);
        double h = g[D - 1] * Tp[D - 1];
#pragma unroll
        for (int k = D - 1; k > CL; --k) h = fma(q, h, g[k - 1] * Tp[k - 1]);
        return h;
    } else {
        return 0.0;
    }
}
template <int D, int CL>
__device__ __forceinline__ double loo_low(const double (&Tp)[D], double q, double v, double s, double top) {
    double h = top;
    if constexpr (CL >= 2) {
        double g[CL];
        cum_g_from<1, CL>(v, s, g);
#pragma unroll
        for (int k = CL; k >= 2; --k) h = fma(q, h, g[k - 1] * Tp[k - 1]);
    }
    h = fma(q, h, Tp[0]);
    return q * h;
}

__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

__device__ __forceinline__ Grid make_grid(int slack, double ctx, double wsum, double wmin, double step0) {
    Grid g;
    g.t_lo = kQuadLo * fast_rcp(slack + wsum);
    const double lowest = slack + ((slack == 0 || ctx == 0.0) ? wmin : 0.0);
    const double range = fast_log((kQuadHi / kQuadLo) * (slack + wsum) * fast_rcp(lowest));
    g.step = step0;
    int N = static_cast<int>(ceil(range / g.step)) + 1;
    if (step0 == kQuadStep && N > 64 && range <= 0.5 * 63.0) { g.step = range / 63.0; N = 64; }
    if (N < 1) N = 1;
    if (N > 4096) N = 4096;
    g.N = N;
    const double estep = g.step == kQuadStep ? 1.5683121854901688 : exp(g.step);      // e^0.45
    g.tail = g.step * g.t_lo * fast_rcp(estep - 1.0);
    g.tail2 = g.step * g.t_lo * g.t_lo * fast_rcp(estep * estep - 1.0);
    return g;
}

// Routed mass of every active token, and the mass left to the slack term.
//
// Tokens are held in decreasing q: first the (at most three, only with more than 8 drafts) heavy ones that keep
// their exact factor, then up to L.nfull tokens with all D cumulants, then the tokens that need four.  A chunk
// of up to 64 quadrature nodes is dealt to the waves (wave w owns nodes w, w + NW, ...), and a wave takes
// its nodes through all three phases without a workgroup barrier:
//   phase 1  lane = (node, token subset): the cumulant sums of its tokens at its node, then a butterfly over
//            the subsets;
//   phase 2  per node: T = exp(z ctx + cumulant series) (times the exact factors of the heavy tokens), the
//            slack integrand, and the node record {t, weight, T_{n-1..n-D}} -> LDS;
//   phase 3  lane = (token, node subset): the leave-one-out coefficient of its token at each of the wave's
//            nodes; the waves' partial sums meet in LDS at the end.
// In: L.trec[] (weights and series terms), L.apd / L.nheavy / L.nfull (set up by solve_program), the grid.
// Out: every wave's partial sums in L.rpart / L.spart / L.r0part.  All waves call it behind a barrier that made
// the weights visible; it contains no workgroup barrier itself.
template <int D>
__device__ __forceinline__ void eval_core_rows(Lds<D>& L, const Grid& gr, int m, int n, double ctx, int slack);

template <int D>
__device__ __forceinline__ void eval_core(Lds<D>& L, const Grid& gr, int m, int n, double ctx, int slack) {
    if constexpr (D <= 8) { eval_core_rows<D>(L, gr, m, n, ctx, slack); return; }
    constexpr int kSW = Lds<D>::kSW, NPW = Lds<D>::kNPW, NS = 64 / NPW;
    constexpr int CL = D < 4 ? D : 4;                          // cumulants of a light token
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int nheavy = (D > 8) ? L.nheavy : 0;
    const int nfull = (D > 4) ? L.nfull : nheavy;              // up to four drafts four cumulants are all there are
    const double t_lo = gr.t_lo, step = gr.step;
    const int N = gr.N;
    for (int i = lane; i < m; i += 64) { L.rpart[wv][i] = 0.0; L.spart[wv][i] = 0.0; }
    double r0 = 0.0;                                       // slack integrand, lanes of token subset 0
    double hacc[kMaxHeavy] = {0.0, 0.0, 0.0}, hacct[kMaxHeavy] = {0.0, 0.0, 0.0};
    const int j = lane & (NPW - 1), tsub = lane / NPW;
    GR_CLK(L, 6);

    for (int c0 = 0; c0 < N; c0 += 64) {
        const int nn = min(64, N - c0);
        const int npw = (nn - wv + kSW - 1) / kSW;          // nodes of this wave in the chunk: c0 + wv + kSW j
        const double t = t_lo * exp(step * static_cast<double>(c0 + wv + kSW * j));
        const double qw = j < npw ? step * t * exp_neg(slack * t, L.e2tab) : 0.0;
        // ---- phase 1: cumulant sums at node j of the tokens of subset tsub
        double K[D];
#pragma unroll
        for (int k = 0; k < D; ++k) K[k] = 0.0;
        if (npw > 0) {
            if constexpr (D > 4) phase1_range<D, D, NS>(K, L.trec, nheavy, nfull, m, tsub, t, L.e2tab);
            phase1_range<D, CL, NS>(K, L.trec, nfull, m, m, tsub, t, L.e2tab);
        }
#pragma unroll
        for (int k = 0; k < D; ++k) {
            if (NS >= 8) K[k] += __shfl_xor(K[k], 8);
            K[k] += __shfl_xor(K[k], 16);
            K[k] += __shfl_xor(K[k], 32);
        }
        GR_CLK(L, 7);
        // ---- phase 2: the node's series T = exp(z ctx + sum_k K_k z^k), every lane of the node alike
        K[0] += ctx;
        double T[D + 1];
        T[0] = 1.0;
        {
            double kK[D];
#pragma unroll
            for (int k = 1; k <= D; ++k) kK[k - 1] = static_cast<double>(k) * K[k - 1];
#pragma unroll
            for (int d = 1; d <= D; ++d) {
                double acc = kK[0] * T[d - 1];
#pragma unroll
                for (int k = 2; k <= d; ++k) acc = fma(kK[k - 1], T[d - k], acc);
                T[d] = acc * (1.0 / d);
            }
        }
        if constexpr (D > 8) {
            // the heavy tokens' exact factors, then each one's leave-one-out coefficient by series division
            double xh[kMaxHeavy];
            for (int hv = 0; hv < nheavy; ++hv) {
                double e[D];
#pragma unroll
                for (int a = 0; a < D; ++a) e[a] = L.trec[hv].e[a];
                xh[hv] = exp_neg(t * L.trec[hv].aw, L.e2tab);
                mul_factor<D>(T, xh[hv], e);
            }
            for (int hv = 0; hv < nheavy; ++hv) {
                double e[D];
#pragma unroll
                for (int a = 0; a < D; ++a) e[a] = L.trec[hv].e[a];
                const double term = (tsub == 0 ? qw : 0.0) * xh[hv] * loo_coeff<D>(T, xh[hv], e, n);
                hacc[hv] += term;
                hacct[hv] = fma(term, t, hacct[hv]);
            }
        }
        {
            NodeRec<D> rec;
            rec.t = t; rec.qw = qw;
            const double tn = pick_series<D, D>(rec, T, n);
            if (tsub == 0) { r0 = fma(qw, tn, r0); L.nrec[wv][j] = rec; }
        }
        wave_lds_sync();
        GR_CLK(L, 8);
        // ---- phase 3
        if constexpr (D > 4) phase3_range<D, D>(L, nheavy, nfull, m, npw, wv, lane);
        phase3_range<D, CL>(L, nfull, m, m, npw, wv, lane);
        wave_lds_sync();                                   // this wave's node records are rewritten by its next chunk
        GR_CLK(L, 9);
    }
    if constexpr (D > 8) {
        for (int hv = 0; hv < nheavy; ++hv) {
            const double a = wave_sum(hacc[hv]), b = wave_sum(hacct[hv]);
            if (lane == 0) { L.rpart[wv][hv] = a; L.spart[wv][hv] = b; }
        }
    }
    {
        const double r0w = wave_sum(r0);
        if (lane == 0) L.r0part[wv] = r0w;
    }
    if (tid == 0) L.work += static_cast<double>(N) * m;
}

// The same evaluation for up to eight drafts (no heavy tokens there), both phases in ONE lane layout: lane = (node j
// of the wave, token subset tsub), token row i of a lane = token NS i + tsub.  The factor x = e^{-t w} of a (node,
// token) pair is computed once, in phase 1, and stays in a register until phase 3 uses it again (NT = kMaxT / NS rows
// per lane; the row loops are unrolled so that the array is indexed by constants).  Phase 3 then needs the node's
// series, which this lane already holds, and the token's q; it ends with a sum over the NPW neighbouring lanes that
// hold the nodes of a subset.  No node records in LDS and no exchange between the phases.
// Rows whose first token is below L.nfull take all D cumulants, the others four.
template <int D>
__device__ __forceinline__ void eval_core_rows(Lds<D>& L, const Grid& gr, int m_, int n_, double ctx, int slack_) {
    constexpr int kSW = Lds<D>::kSW, NPW = Lds<D>::kNPW, NS = 64 / NPW, NT = kMaxT / NS;
    constexpr int CL = D < 4 ? D : 4;
    static_assert(D <= 8 && NPW == 8 && NT % 2 == 0, "rows are taken two at a time; eight node lanes per subset");
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    // the sizes are the same in every lane; said so, the row guards below are scalar branches, not lane masks
    const int m = __builtin_amdgcn_readfirstlane(m_), n = __builtin_amdgcn_readfirstlane(n_);
    const int slack = __builtin_amdgcn_readfirstlane(slack_);
    const int nfull = (D > 4) ? __builtin_amdgcn_readfirstlane(L.nfull) : 0;
    const double t_lo = gr.t_lo, step = gr.step;
    const int N = __builtin_amdgcn_readfirstlane(gr.N);
    const int j = lane & (NPW - 1), tsub = lane / NPW;
    for (int i = lane; i < kMaxT; i += 64) { L.rpart[wv][i] = 0.0; L.spart[wv][i] = 0.0; }
    double r0 = 0.0;                                       // slack integrand, lanes of token subset 0
    GR_CLK(L, 6);

    for (int c0 = 0; c0 < N; c0 += 64) {
        const int nn = min(64, N - c0);
        const int npw = (nn - wv + kSW - 1) / kSW;          // nodes of this wave in the chunk: c0 + wv + kSW j
        const double t = t_lo * exp(step * static_cast<double>(c0 + wv + kSW * j));
        const double qw = j < npw ? step * t * exp_neg(slack * t, L.e2tab) : 0.0;
        // ---- phase 1: cumulant sums at this lane's node over the tokens of its subset
        double K[D], xs[NT];
#pragma unroll
        for (int k = 0; k < D; ++k) K[k] = 0.0;
        // the weights of a pair of rows are requested one pair ahead: they head the longest chain (the exponential)
        double awa = L.trec[tsub].aw, awb = L.trec[tsub + NS].aw;
#pragma unroll
        for (int i = 0; i < NT; i += 2) {
            xs[i] = 0.0; xs[i + 1] = 0.0;
            if (NS * i < m) {
                const int a = NS * i + tsub, b = a + NS;
                const TokRec<D>& ra = L.trec[a];               // the records behind the last token have x = 0
                const TokRec<D>& rb = L.trec[b];
                const double ya = t * awa, yb = t * awb;
                if (i + 2 < NT) {
                    awa = L.trec[b + NS].aw;
                    awb = L.trec[b + 2 * NS].aw;
                }
                double x0, x1;
                exp_neg2(ya, yb, L.e2tab, x0, x1);
                if (D > 4 && NS * i < nfull) { phase1_token<D, D>(K, ra, x0); phase1_token<D, D>(K, rb, x1); }
                else { phase1_token<D, CL>(K, ra, x0); phase1_token<D, CL>(K, rb, x1); }
                xs[i] = x0; xs[i + 1] = x1;
            }
        }
#pragma unroll
        for (int k = 0; k < D; ++k) {
            if (NS >= 8) K[k] += __shfl_xor(K[k], 8);
            K[k] += __shfl_xor(K[k], 16);
            K[k] += __shfl_xor(K[k], 32);
        }
        GR_CLK(L, 7);
        // ---- phase 2: the node's series T = exp(z ctx + sum_k K_k z^k), every lane of the node alike
        K[0] += ctx;
        double T[D + 1];
        T[0] = 1.0;
        {
            double kK[D];
#pragma unroll
            for (int k = 1; k <= D; ++k) kK[k - 1] = static_cast<double>(k) * K[k - 1];
#pragma unroll
            for (int d = 1; d <= D; ++d) {
                double acc = kK[0] * T[d - 1];
#pragma unroll
                for (int k = 2; k <= d; ++k) acc = fma(kK[k - 1], T[d - k], acc);
                T[d] = acc * (1.0 / d);
            }
        }
        double Tp[D];                                      // quadrature weight x T_{n-k} / k!
        {
            NodeRec<D> rec;
            const double tn = pick_series<D, D>(rec, T, n);
            if (tsub == 0) r0 = fma(qw, tn, r0);
            double invf = qw;
#pragma unroll
            for (int k = 1; k <= D; ++k) { invf *= 1.0 / k; Tp[k - 1] = rec.Tr[k - 1] * invf; }
        }
        GR_CLK(L, 8);
        // ---- phase 3: the leave-one-out coefficient of every pair, summed over the nodes of the wave.  The sums over
        // the eight node lanes of a subset: the first step (lane k with lane 7 - k) also parts the two sums, R to
        // lanes 0-3 and its t-weighted companion S to lanes 4-7, so that the other two steps move one value, not two.
        double qna = L.trec[tsub].e[0], qnb = L.trec[tsub + NS].e[0];
        const bool upper = (NPW == 8) && j >= 4;
        double* const part = upper ? &L.spart[wv][0] : &L.rpart[wv][0];
#pragma unroll
        for (int i = 0; i < NT; i += 2) {
            if (NS * i < m) {
                const int a = NS * i + tsub, b = a + NS;            // b <= kMaxT - 1: sums of rows past the last token are 0
                double olda = 0.0, oldb = 0.0;
                if ((j & 3) == 0) { olda = part[a]; oldb = part[b]; }
                const double qa = qna, qb = qnb;
                if (i + 2 < NT) {
                    qna = L.trec[b + NS].e[0];
                    qnb = L.trec[b + 2 * NS].e[0];
                }
                const double x0 = xs[i], x1 = xs[i + 1];
                const double v0 = fma(-x0, x0, x0), s0 = fma(-2.0, x0, 1.0), v1 = fma(-x1, x1, x1), s1 = fma(-2.0, x1, 1.0);
                double ta = 0.0, tb = 0.0;
                if (D > CL && NS * i < nfull) { ta = loo_top<D, CL>(Tp, qa, v0, s0); tb = loo_top<D, CL>(Tp, qb, v1, s1); }
                const double ca = loo_low<D, CL>(Tp, qa, v0, s0, ta), cb = loo_low<D, CL>(Tp, qb, v1, s1, tb);
                const double ra_ = xs[i] * ca, rb_ = xs[i + 1] * cb;
                const double sa_ = ra_ * t, sb_ = rb_ * t;
                double ka = upper ? sa_ : ra_, kb = upper ? sb_ : rb_;
                ka += dpp_move<kDppHalfMirror>(upper ? ra_ : sa_);
                kb += dpp_move<kDppHalfMirror>(upper ? rb_ : sb_);
                ka += dpp_move<kDppXor1>(ka); kb += dpp_move<kDppXor1>(kb);
                ka += dpp_move<kDppXor2>(ka); kb += dpp_move<kDppXor2>(kb);
                if ((j & 3) == 0) { part[a] = olda + ka; part[b] = oldb + kb; }
            }
        }
        GR_CLK(L, 9);
    }
    {
        const double r0w = wave_sum(r0);
        if (lane == 0) L.r0part[wv] = r0w;
    }
    if (tid == 0) L.work += static_cast<double>(N) * m;
}

// The routed mass R and its t-weighted companion S of token `tok` from the waves' partial sums (behind the
// barrier that follows eval_core), and the slack mass.
template <int D>
__device__ __forceinline__ void token_sums(const Lds<D>& L, const Grid& gr, int tok, double fact, double& R, double& S) {
    constexpr int kSW = Lds<D>::kSW;
    const double rfact = fast_rcp(fact);
    double r = L.apd[tok] * gr.tail * rfact, sq = L.apd[tok] * gr.tail2 * rfact;
#pragma unroll
    for (int w2 = 0; w2 < kSW; ++w2) { r += L.rpart[w2][tok]; sq += L.spart[w2][tok]; }
    const double w = L.trec[tok].aw;
    R = r * w * fact;
    S = sq * w * w * fact;
}
template <int D>
__device__ __forceinline__ double slack_mass(const Lds<D>& L, const Grid& gr, int n, double atot, double fact, int slack) {
    constexpr int kSW = Lds<D>::kSW;
    double r0all = 0.0;
#pragma unroll
    for (int w2 = 0; w2 < kSW; ++w2) r0all += L.r0part[w2];
    return (r0all * fact + ipow(atot, n) * gr.tail) * slack;
}

// Workgroup-wide evaluation (the Newton fallback's): every thread passes the log weight of its own token and gets
// that token's routed mass back (also left in L.aR); returns the slack mass.  All threads call it.
struct Routed { double R0, R, S; };
template <int D>
__device__ __forceinline__ Routed routed_eval(Lds<D>& L, int& par, int m, int n, double ctx, int slack, double qsum, double fact, double alpha) {
    const int tid = threadIdx.x;
    double w = 0.0;
    if (tid < m) { w = exp(alpha); L.trec[tid].aw = w; }
    double a[2] = {wave_sum(tid < m ? w : 0.0), wave_min(tid < m ? w : 1e300)};
    wg_reduce<2>(L, par, a, {kOpSum, kOpMin});              // its barrier also publishes the weights
    const Grid gr = make_grid(slack, ctx, a[0], a[1], kQuadStep);
    eval_core<D>(L, gr, m, n, ctx, slack);
    __syncthreads();
    Routed out;
    out.R = 0.0; out.S = 0.0;
    if (tid < m) { token_sums<D>(L, gr, tid, fact, out.R, out.S); L.aR[tid] = out.R; }
    out.R0 = slack_mass<D>(L, gr, n, ctx + qsum, fact, slack);
    GR_CLK(L, 10);
    return out;
}

// One evaluation and the stopping measure: max_i | log(target_i / routed_i) - common term |, where the
// common term is log(slack_target / slack mass) with slack, log(sum target / sum routed) without
// (the latter is zero in exact arithmetic and removes the common quadrature error).  Per-token quantities are
// those of the calling thread's token: alpha and target in, f = log(target / routed) - common term, R and S out.
struct Defect { double err, f, R, S, rsum, R0; };
template <int D>
__device__ __forceinline__ Defect defect_eval(Lds<D>& L, int& par, int m, int n, double ctx, int slack, double slack_target, double qsum,
                                              double tsum, double fact, double alpha, double target) {
    const int tid = threadIdx.x;
    Defect d;
    {
        const Routed r = routed_eval<D>(L, par, m, n, ctx, slack, qsum, fact, alpha);
        d.R0 = r.R0; d.R = r.R; d.S = r.S;
    }
    double g = 0.0;
    if (tid < m) { g = fast_log(target / d.R); if (!(g == g)) g = 1e301; }
    double a[3] = {wave_sum(tid < m ? d.R : 0.0), wave_max(tid < m ? g : -1e300), wave_min(tid < m ? g : 1e300)};
    wg_reduce<3>(L, par, a, {kOpSum, kOpMax, kOpMin});
    d.rsum = a[0];
    const double gmax = a[1], gmin = a[2];
    const double lc = fast_log(slack ? d.R0 / slack_target : d.rsum / tsum);
    d.f = tid < m ? g + lc : 0.0;
    double worst = fmax(fabs(gmax + lc), fabs(gmin + lc));
    if (!(worst == worst)) worst = 1e301;                  // NaN: treated as "no finite point"
    if (!(gmax < 1e300) || !(gmin > -1e300)) worst = 1e301;
    d.err = worst;
    GR_CLK(L, 11);
    return d;
}

// Damped Newton iteration on routed(alpha) = target with a finite-difference Jacobian (the Hessian of
// Theta_T / Phi_T in alpha), for programs on which the fixed-point iteration is slow (a target that
// nearly exhausts the tuples containing its token).  One step costs one evaluation per variable, so
// it only takes over when the mixed iteration has used up its budget.  Without slack the last weight
// is pinned (the system is singular along the common shift).  Starts from L.aal.
// J: this row's scratch in HBM, kMaxT rows of kMaxT + 1 doubles (the last column is the right-hand side).
// The cap counts the evaluations of this program only (`evals0` = the row's count when the program began).
template <int D>
__device__ int newton_program(Lds<D>& L, int& par, double* J, int m, int n, double ctx, int slack, double slack_target, double qsum,
                              double tsum, double fact, double rel_tol, int max_evals, int* evals, int evals0) {
    constexpr int kSW = Lds<D>::kSW;
    const int tid = threadIdx.x;
    const int nfree = slack ? m : m - 1;
    constexpr int LD = kMaxT + 1;
    constexpr double kFd = 1e-6;
    const double target = tid < m ? L.at[tid] : 0.0;
    Defect dd = defect_eval<D>(L, par, m, n, ctx, slack, slack_target, qsum, tsum, fact, tid < m ? L.aal[tid] : 0.0, target);
    double err = dd.err, rsum = dd.rsum, R0 = dd.R0, f = dd.f;
    *evals += 1;
    while (err > rel_tol && *evals - evals0 < max_evals && err < 1e300) {
        if (tid < m) { L.nR[tid] = L.aR[tid]; L.af[tid] = f; }
        // common ratio routed/target over all vertices, the slack vertex included: Newton aims at
        // routed_j = ratio * target_j, which is what the stopping measure asks for
        const double ratio = slack ? (rsum + R0) / (tsum + slack_target) : rsum / tsum;
        __syncthreads();
        for (int k = 0; k < nfree; ++k) {
            if (tid == k) L.aal[k] += kFd;
            __syncthreads();
            const Routed rk = routed_eval<D>(L, par, m, n, ctx, slack, qsum, fact, tid < m ? L.aal[tid] : 0.0);
            if (tid < nfree) J[tid * LD + k] = (rk.R - L.nR[tid]) / kFd;
            if (tid == k) L.aal[k] -= kFd;
            __syncthreads();
        }
        *evals += nfree;
        if (tid < nfree) { J[tid * LD + kMaxT] = L.at[tid] * ratio - L.nR[tid]; L.nused[tid] = 0; L.ncolof[tid] = -1; L.nstep[tid] = 0.0; }
        __syncthreads();
        // Gauss-Jordan with partial pivoting: thread r owns row r
        for (int c = 0; c < nfree; ++c) {
            const double mag = (tid < nfree && !L.nused[tid]) ? fabs(J[tid * LD + c]) : -1.0;
            const double best = block_max<kSW>(mag, L.redn);
            if (!(best > 0.0)) continue;                   // no pivot left in this column: its step stays 0
            const int who = static_cast<int>(block_min<kSW>(mag == best ? static_cast<double>(tid) : 1e9, L.redn));
            const double piv = J[who * LD + c];
            if (tid < nfree && tid != who) {
                const double fct = J[tid * LD + c] / piv;
                for (int jc = c; jc < nfree; ++jc) J[tid * LD + jc] -= fct * J[who * LD + jc];
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
        const double smax = block_max<kSW>(tid < nfree ? fabs(L.nstep[tid]) : 0.0, L.redn);
        if (!(smax < 1e300)) break;
        const double clip = smax > 2.0 ? 2.0 / smax : 1.0;
        // slope of the objective along the step: grad . d with grad_j = routed_j - ratio * target_j
        double slope0 = block_sum<kSW>(tid < nfree ? (L.nR[tid] - L.at[tid] * ratio) * clip * L.nstep[tid] : 0.0, L.redn);
        if (!(slope0 < 0.0)) {
            // not a descent direction (noise in the difference quotients): take the plain
            // fixed-point step instead, which always is one
            if (tid < nfree) L.nstep[tid] = L.af[tid] / clip;
            __syncthreads();
            slope0 = block_sum<kSW>(tid < nfree ? (L.nR[tid] - L.at[tid] * ratio) * L.af[tid] : 0.0, L.redn);
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
            dd = defect_eval<D>(L, par, m, n, ctx, slack, slack_target, qsum, tsum, fact, tid < m ? L.aal[tid] : 0.0, target);
            err2 = dd.err; rsum = dd.rsum; R0 = dd.R0; f = dd.f;
            *evals += 1;
            const double ratio2 = slack ? (rsum + R0) / (tsum + slack_target) : rsum / tsum;
            const double slope = block_sum<kSW>(tid < nfree ? (L.aR[tid] - L.at[tid] * ratio2) * clip * L.nstep[tid] : 0.0, L.redn);
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

// The mixing step of one iteration, by wave 0 alone behind the barrier that follows the evaluation.  Compiled as a
// function of its own (not inlined) so that its values do not compete for registers with the evaluator's series.
// The uniform solver state travels in MixState; per-token values live in LDS (see solve_program).
struct MixState { int hcount, plain, since, odds; double best_err, cap; };
template <int D>
__device__ __attribute__((noinline)) MixState mix_step(MixState st, Grid gr, int it, int m, int n, int slack, double ctx, double slack_target,
                                                      double tsum, double atot, double fact, double rel_tol, int evals) {
    Lds<D>& L = *reinterpret_cast<Lds<D>*>(gr_lds_raw);
    const int tid = threadIdx.x, lane = tid & 63;
    int hcount = st.hcount, plain = st.plain, since = st.since;
    double best_err = st.best_err, cap = st.cap;
    const int tk[2] = {lane, lane + 64};
    const bool on[2] = {tk[0] < m, tk[1] < m};
    double R[2] = {0.0, 0.0}, S[2] = {0.0, 0.0}, g[2] = {0.0, 0.0}, al[2] = {0.0, 0.0};
#pragma unroll
    for (int u = 0; u < 2; ++u) if (on[u]) {
        R[u] = L.aR[tk[u]]; S[u] = L.aS[tk[u]]; g[u] = L.ag[tk[u]];
        al[u] = L.aal[tk[u]];
    }
    GR_CLK(L, 18);
    // stopping measure: max_i | log(target_i / routed_i) - common term |, the common term log(slack_target / slack
    // mass) with slack, log(sum target / sum routed) without (zero in exact arithmetic: it removes the common
    // quadrature error)
    const double rd[3] = {L.ared[0][0] + L.ared[1][0], fmax(L.ared[0][1], L.ared[1][1]), fmin(L.ared[0][2], L.ared[1][2])};
    GR_CLK(L, 19);
    const double lc = slack ? L.alc : fast_log(rd[0] * fast_rcp(tsum));
    double err = fmax(fabs(rd[1] + lc), fabs(rd[2] + lc));
    if (!(err == err) || !(rd[1] < 1e300) || !(rd[2] > -1e300)) err = 1e301;      // NaN or infinite: "no finite point"
#ifdef GR_PHASE_CLOCKS
    if (tid == 0 && evals <= 24) L.errlog[evals - 1] = err;
#endif
    GR_CLK(L, 11);
    // The fixed-point step log(target / routed) treats the routed mass as proportional to the
    // weight; its true logarithmic derivative is (R - S) / R with S = w^2 int t ... (the share a
    // token loses to itself), so the step of each coordinate is stretched by R / (R - S), at most
    // `cap`.  The stretched iteration is no longer monotone: when kStall iterations bring no
    // better point it returns to the best one with half the cap; at cap 1 (the plain step, whose
    // stopping measure need not fall at every step) it is left alone.
    double f[2], ratio[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        f[u] = on[u] ? g[u] + lc : 0.0;
        const double d = R[u] - S[u];
        ratio[u] = (on[u] && d > 0.0) ? fmin(R[u] * fast_rcp(d), 1e30) : (on[u] ? 1e30 : 1.0);
    }
    // A token whose target nearly exhausts P = Pr[token drawn] (in the targets' units) can saturate: its routed mass
    // hardly answers to its weight, log(target / R) flattens out and the stretched step crawls (the start weights
    // leave such a token at log 2 from its target, and every other token has settled long before it has).  What is
    // linear in its log weight there is the log odds R / (P - R) (the single-draft rule is their fixed point), so
    // while the iteration is far from its end such a token steps by the difference of the log odds instead, the
    // stretch changing with it: d log(R / (P - R)) = (R - S) / R * P / (P - R) d log w.  The tokens are chosen once,
    // at the program's first evaluation (a token that starts near its target is better off with the plain form,
    // and a form that changes from one iteration to the next spoils the mixing); below kOddsUntil the plain form
    // takes over for good: the factor P / (P - R) would amplify the error of the quadrature.
    int odds = st.odds;                                // 0: off, 1: on, 2: on and some token of this program steps on its odds
    if (odds && err < kOddsUntil) odds = 0;
    if (odds) {
        bool sel[2]; double P[2] = {1.0, 1.0}, tg[2] = {0.0, 0.0};
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            if (on[u]) { P[u] = L.apd[tk[u]]; tg[u] = L.at[tk[u]]; }
            if (it == 1 && on[u]) L.aodds[tk[u]] = (tg[u] > kOddsFrom * P[u] && tg[u] < kOddsTo * P[u] && fabs(f[u]) > kOddsFirst) ? 1 : 0;
            sel[u] = on[u] && L.aodds[on[u] ? tk[u] : 0] != 0 && R[u] < P[u];
        }
        const bool some = __any(sel[0] || sel[1]);
        if (it == 1) odds = some ? 2 : 0;              // a program without such a token never looks again
        if (some) {
#pragma unroll
            for (int u = 0; u < 2; ++u) if (sel[u]) {
                const double room = P[u] - R[u];
                f[u] += fast_log(room * fast_rcp(P[u] - tg[u]));
                ratio[u] = fmax(ratio[u] * room * fast_rcp(P[u]), 1.0);
            }
        }
    }
    bool stop = false;
    if (err <= rel_tol) {
        if (lane == 0) L.ctl_result = 0;
        stop = true;
    } else if (!(err < 1e300) || err > 100.0 * best_err) {
        // a mixed step went astray: back to the best point, unmixed steps for a while
        if (!(best_err < 1e300)) stop = true;          // no finite point seen: give up on this program
#pragma unroll
        for (int u = 0; u < 2; ++u) if (on[u]) { al[u] = L.aBest[tk[u]]; f[u] = L.fBest[tk[u]]; ratio[u] = L.rBest[tk[u]]; }
        hcount = 0; plain = 20; since = 0;
    } else if (err < best_err) {
        best_err = err; since = 0;
#pragma unroll
        for (int u = 0; u < 2; ++u) if (on[u]) { L.aBest[tk[u]] = al[u]; L.fBest[tk[u]] = f[u]; L.rBest[tk[u]] = ratio[u]; }
    } else if (cap > 1.0 && ++since >= kStall) {
#pragma unroll
        for (int u = 0; u < 2; ++u) if (on[u]) { al[u] = L.aBest[tk[u]]; f[u] = L.fBest[tk[u]]; ratio[u] = L.rBest[tk[u]]; }
        hcount = 0; since = 0;
        cap = fmax(1.0, 0.5 * cap);
    }
    if (stop) {
        if (lane == 0) { L.ctl_go = 0; L.ctl_bestok = best_err < 1e300 ? 1 : 0; }
        return st;
    }
#pragma unroll
    for (int u = 0; u < 2; ++u) f[u] *= fmin(ratio[u], cap);
    GR_CLK(L, 16);
    const int cur = it % kHist;
    const int navail = min(hcount, kCols);             // stored vectors since the history was last dropped
    const int ncol = plain > 0 ? 0 : navail;
    if (plain > 0) --plain;
    // inner products of the new residual vector with itself and the stored ones, and the longest plain step
    double hf[kCols][2], ha[kCols][2];
    double ex[kHist + 1];
    ex[0] = f[0] * f[0] + f[1] * f[1];
    ex[kHist] = fmax(fabs(f[0]), fabs(f[1]));
#pragma unroll
    for (int c = 0; c < kCols; ++c) {
        const int slot = (cur - 1 - c + 2 * kHist) % kHist;
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            hf[c][u] = (on[u] && c < navail) ? L.Hf[slot][tk[u]] : 0.0;
            ha[c][u] = (on[u] && c < navail) ? L.Ha[slot][tk[u]] : 0.0;
        }
        ex[1 + c] = f[0] * hf[c][0] + f[1] * hf[c][1];
    }
    wave_reduce_many<kHist + 1>(ex, {kOpSum, kOpSum, kOpSum, kOpSum, kOpSum, kOpMax});
    GR_CLK(L, 17);
    double stepv[2] = {f[0], f[1]};
    if (ncol >= 1) {
        // normal equations of  min || f - dF gamma ||  with dF_c = f - f_c:  <dF_a, dF_b> and <dF_a, f> from the
        // inner products (the new vector's are in ex, the older ones in L.pm: lane 4a + b fetches entry (a, b));
        // Gaussian elimination without pivoting (symmetric positive definite after the ridge), in registers
        double old;
        {
            const int la = (lane >> 2) & 3, lb = lane & 3;
            old = L.pm[(cur - 1 - la + 2 * kHist) % kHist][(cur - 1 - lb + 2 * kHist) % kHist];
        }
        double Gm[kCols][kCols + 1];
#pragma unroll
        for (int a2 = 0; a2 < kCols; ++a2) {
#pragma unroll
            for (int b2 = 0; b2 < kCols; ++b2) Gm[a2][b2] = (ex[0] - ex[1 + a2]) - (ex[1 + b2] - read_lane(old, 4 * a2 + b2));
            Gm[a2][kCols] = ex[0] - ex[1 + a2];
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
                double inv = __builtin_amdgcn_rcp(Gm[c][c]);          // reciprocal: two Newton steps from the hardware estimate
                inv = inv * fma(-Gm[c][c], inv, 2.0);
                inv = inv * fma(-Gm[c][c], inv, 2.0);
                pivinv[c] = inv;
#pragma unroll
                for (int r = c + 1; r < kCols; ++r) {
                    if (r < ncol) {
                        const double fct = Gm[r][c] * inv;
#pragma unroll
                        for (int jc = c + 1; jc <= kCols; ++jc) Gm[r][jc] = fma(-fct, Gm[c][jc], Gm[r][jc]);
                    }
                }
            }
        }
        double gam[kCols];
#pragma unroll
        for (int c = kCols - 1; c >= 0; --c) {
            double sacc = Gm[c][kCols];
#pragma unroll
            for (int jc = c + 1; jc < kCols; ++jc) if (jc < ncol) sacc = fma(-Gm[c][jc], gam[jc], sacc);
            gam[c] = (c < ncol) ? sacc * pivinv[c] : 0.0;
        }
        double gnorm = 0.0;
#pragma unroll
        for (int c = 0; c < kCols; ++c) gnorm += fabs(gam[c]);
        const bool solved = good && gnorm < 1e300;
        double cand[2] = {f[0], f[1]};
#pragma unroll
        for (int c = 0; c < kCols; ++c)
#pragma unroll
            for (int u = 0; u < 2; ++u) if (c < ncol) cand[u] -= ((al[u] - ha[c][u]) + (f[u] - hf[c][u])) * gam[c];
        const double cmax = wave_max(fmax(on[0] ? fabs(cand[0]) : 0.0, on[1] ? fabs(cand[1]) : 0.0));
        // a mixed step longer than 3 in log weight is cut to that length (the same cap as the
        // Newton fallback); a failed solve drops the history
        if (solved && cmax < 1e300) {
            const double cut = cmax > 3.0 ? 3.0 * fast_rcp(cmax) : 1.0;
            stepv[0] = cand[0] * cut; stepv[1] = cand[1] * cut;
        } else hcount = 0;
    } else {                                           // a plain step: the same cap on its length
        const double fmx = ex[kHist];
        if (fmx > 3.0) { const double cut = 3.0 * fast_rcp(fmx); stepv[0] = f[0] * cut; stepv[1] = f[1] * cut; }
    }
    GR_CLK(L, 20);
    // the new vector takes slot `cur` of the history (its inner products are read again next iteration)
    if (lane <= kCols) {
        const int slot = lane == 0 ? cur : (cur - lane + 2 * kHist) % kHist;
        double val = ex[0];                             // ex[lane] without indexing registers by a variable
#pragma unroll
        for (int c = 1; c <= kCols; ++c) if (lane == c) val = c - 1 < navail ? ex[c] : 0.0;
        L.pm[cur][slot] = val; L.pm[slot][cur] = val;
    }
    double ws = 0.0, wm = 1e300, amax = -1e300;
#pragma unroll
    for (int u = 0; u < 2; ++u) if (on[u]) {
        L.Ha[cur][tk[u]] = al[u]; L.Hf[cur][tk[u]] = f[u];
        al[u] += stepv[u];
        amax = fmax(amax, al[u]);
    }
    if (!slack) amax = wave_max(amax); else amax = 0.0;   // without slack only differences of log weights matter
#pragma unroll
    for (int u = 0; u < 2; ++u) if (on[u]) {
        al[u] -= amax;
        const double w = exp_signed(al[u], L.e2tab);
        L.aal[tk[u]] = al[u]; L.trec[tk[u]].aw = w; ws += w; wm = fmin(wm, w);
    }
    ws = wave_sum(ws); wm = wave_min(wm);
    if (lane == 0) {
        L.ctl_grid = make_grid(slack, ctx, ws, wm, kQuadStep); L.ctl_bestok = best_err < 1e300 ? 1 : 0;
    }
    ++hcount;
    st.hcount = hcount; st.plain = plain; st.since = since; st.odds = odds; st.best_err = best_err; st.cap = cap;
    GR_CLK(L, 12);
    return st;
}

// Solve one program by iterative scaling with Anderson mixing.  Returns 0 when converged.
// In: L.aq, L.at (targets, already scaled to the tuple mass), L.aal (start log weights), each written by the
// thread of its token; qsum = sum aq, tsum = sum at.
// Out: L.aal.  `evals` counts evaluator calls (summed over the row's programs; max_iter caps this program's).
template <int D>
__device__ __forceinline__ int solve_program(Lds<D>& L, int& par, double* newton_ws, int m, int n, double ctx, int slack, double slack_target,
                             double qsum, double tsum, double rel_tol, int max_iter, int* evals) {
    constexpr int kSW = Lds<D>::kSW;
    const int tid = threadIdx.x;
    const int evals0 = *evals;
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
        return wg_sum(L, par, static_cast<double>(stuck)) > 0.0 ? 1 : 0;
    }
    const double atot = ctx + qsum;
    int heavy = 0, full = 0;
    if (tid < m) {
        // per-token series of e^{zq}: q^k / k! for k <= n (terms beyond z^n never reach the z^n coefficient)
        const double q = L.aq[tid];
        double e = 1.0;
#pragma unroll
        for (int a = 1; a <= D; ++a) {
            e = e * q * (1.0 / a);
            L.trec[tid].e[a - 1] = a <= n ? e : 0.0;
        }
        L.trec[tid].pad = 0.0;
        L.apd[tid] = pow_diff(atot, q, n);
        // With more than 8 drafts the cumulant series of a token that dominates the draw mass loses digits to
        // cancellation: the (at most three) tokens above kHeavyShare keep their exact factor instead.
        heavy = (D > 8 && q > kHeavyShare * atot) ? 1 : 0;
        // A token needs only four cumulants when the u^5 and later terms of its factor cannot change the z^n
        // coefficient by more than 1e-11 relative: C(n-1, 4) (q/atot)^4 / 5 < 1e-11 (always, up to four drafts).
        const double r = q / atot;
        double binom = 1.0;
        for (int c = 1; c <= 4; ++c) binom = binom * (n - c) / c;         // C(n-1, 4)
        full = (D > 4 && !(binom * r * r * r * r / 5.0 < 1e-11)) ? 1 : 0;
    }
    if (tid < 32) L.e2tab[tid] = exp2(-static_cast<double>(tid) / 32.0);
    if (tid >= m && tid < kMaxT + 4) {                     // every record behind the last token: x = 0, no mass
        TokRec<D>& z = L.trec[tid];
        z.aw = 1e300; z.pad = 0.0;
#pragma unroll
        for (int a = 0; a < D; ++a) z.e[a] = 0.0;
    }
    if (D > 4) {
        // tokens are in decreasing q: the heavy ones are the first nh, those with all cumulants the first nf
        double a[2] = {wave_sum(static_cast<double>(heavy)), wave_sum(static_cast<double>(full))};
        wg_reduce<2>(L, par, a, {kOpSum, kOpSum});
        const int nh = static_cast<int>(a[0]), nf = static_cast<int>(a[1]);
        if (tid == 0) { L.nheavy = nh < kMaxHeavy ? nh : kMaxHeavy; L.nfull = nf > L.nheavy ? nf : L.nheavy; }
    }
    __syncthreads();
    GR_CLK(L, 5);
    double fact = 1.0;
    for (int i = 2; i <= n; ++i) fact *= i;
    const int mix_iters = (max_iter > kMixBudget + m) ? kMixBudget + m : max_iter;
    const int wvi = tid >> 6, lane = tid & 63;
    // The iteration is steered by wave 0 alone (lane l holds tokens l and l + 64, so every reduction over the
    // tokens is a wave reduction and the mixing needs no workgroup exchange); all waves evaluate.  Per
    // iteration: barrier, evaluation by all waves, barrier, mixing step by wave 0 (the others wait at the next
    // barrier).  Wave 0 hands over through L.ctl_*: whether to go on, and the quadrature grid of the new weights.
    // Wave-0 state: uniform scalars in registers, per-token values in LDS (L.aal, L.at, the best point, the last
    // kHist iterates and stretched residuals by slot, L.pm = inner products of the stored residual vectors).
    MixState st;
    st.hcount = 0; st.plain = 0; st.since = 0; st.odds = 1; st.best_err = 1e300; st.cap = kStretch;
    const int tk[2] = {lane, lane + 64};
    const bool on[2] = {wvi == 0 && tk[0] < m, wvi == 0 && tk[1] < m};
    if (wvi == 0) {
        double ws = 0.0, wm = 1e300, amax = -1e300;
        if (!slack) {
#pragma unroll
            for (int u = 0; u < 2; ++u) if (on[u]) amax = fmax(amax, L.aal[tk[u]]);
            amax = wave_max(amax);
        } else amax = 0.0;
#pragma unroll
        for (int u = 0; u < 2; ++u) if (on[u]) {
            const double al = L.aal[tk[u]] - amax;
            const double w = exp_signed(al, L.e2tab);
            L.aal[tk[u]] = al; L.trec[tk[u]].aw = w; ws += w; wm = fmin(wm, w);
        }
        ws = wave_sum(ws); wm = wave_min(wm);
        if (lane == 0) { L.ctl_go = 1; L.ctl_result = 1; L.ctl_bestok = 0; L.ctl_grid = make_grid(slack, ctx, ws, wm, kQuadStep); }
    }
    for (int it = 1; it <= mix_iters; ++it) {
        __syncthreads();                                   // the weights and L.ctl of this iteration are in place
        if (!L.ctl_go) break;
        const Grid gr = L.ctl_grid;
        eval_core<D>(L, gr, m, n, ctx, slack);
        *evals += 1;
        __syncthreads();                                   // every wave's partial sums are in place
        GR_CLK(L, 10);
        // one token per thread: its routed mass R, the companion S and log(target / R); one thread the slack mass.
        // Done here by the first waves side by side, not by the mixing wave for two tokens per lane.
        if (tid < kMaxT) {                                 // the first two waves, whole
            double R = 0.0, S = 0.0, g = 0.0;
            if (tid < m) {
                token_sums<D>(L, gr, tid, fact, R, S);
                g = fast_log(L.at[tid] * fast_rcp(R));
                if (!(g == g)) g = 1e301;
                L.aR[tid] = R; L.aS[tid] = S; L.ag[tid] = g;
            }
            double a3[3] = {tid < m ? R : 0.0, tid < m ? g : -1e300, tid < m ? g : 1e300};
            wave_reduce_many<3>(a3, {kOpSum, kOpMax, kOpMin});
            if (lane == 0) { L.ared[wvi][0] = a3[0]; L.ared[wvi][1] = a3[1]; L.ared[wvi][2] = a3[2]; }
        } else if (tid == kMaxT) {
            const double R0 = slack_mass<D>(L, gr, n, atot, fact, slack);
            L.aR0 = R0;
            if (slack) L.alc = fast_log(R0 * fast_rcp(slack_target));
        }
        __syncthreads();
        if (wvi != 0) continue;
        st = mix_step<D>(st, gr, it, m, n, slack, ctx, slack_target, tsum, atot, fact, rel_tol, *evals);
    }
    __syncthreads();
    int result = L.ctl_result;
    const bool bestok = L.ctl_bestok != 0;
    GR_CLK(L, 12);
    if (result != 0 && mix_iters < max_iter && bestok) {
        if (tid < m) L.aal[tid] = L.aBest[tid];
        __syncthreads();
        result = newton_program<D>(L, par, newton_ws, m, n, ctx, slack, slack_target, qsum, tsum, fact, rel_tol, max_iter, evals, evals0);
        GR_CLK(L, 13);
    }
    return result;
}

// Build the active list of one program: the support positions in [lo, hi) that belong to T and have
// a positive target, in decreasing q (L.ordq lists the positions of H* and of the rest in that
// order).  Returns m (possibly > kMaxT, in which case nothing was written beyond kMaxT).
template <class LdsT>
__device__ int compact_active(LdsT& L, int lo, int hi, int kk) {
    constexpr int kSW = LdsT::kSW;
    const int tid = threadIdx.x;
    const int j = tid < kk ? L.ordq[tid] : -1;           // kk <= KS <= kST
    const int on = (j >= lo && j < hi && L.inT[j] && L.tgt[j] > 0.0) ? 1 : 0;
    // inclusive scan of `on` over the workgroup
    int incl = on;
    for (int o = 1; o < 64; o <<= 1) { const int up = __shfl_up(incl, o); if ((tid & 63) >= o) incl += up; }
    int* wtot = reinterpret_cast<int*>(L.redn);
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
__global__ __launch_bounds__(kThreadsOf<D>) void solve_kernel(SolveParams sp) {
    constexpr int kST = Lds<D>::kST, kSW = Lds<D>::kSW;
    Lds<D>& L = *reinterpret_cast<Lds<D>*>(gr_lds_raw);
    const int tid = threadIdx.x;
    const int row = blockIdx.x;
    const int n = sp.n, V = sp.V;
    RowInfo info;
    info.support = 0; info.h = 0; info.status = GR_ROW_OK; info.iterations = 0;
    info.alpha_star = 0.0; info.res_total = 0.0; info.p_total = 0.0; info.q_total = 0.0; info.node_tokens = 0.0; info.p_ref = 0.0; info.inv_temp = 0.0; info.q_ref = 0.0;

    // ---- merge the slices
    int total = 0, bad = 0;
    double ptot = 0.0, qtot = 0.0;
    double p_ref = 0.0, inv_temp = 0.0, inv_temp_q = 0.0;
    if (sp.logits) {
        // rows given as logits: the slices' softmax sums are brought to the row's largest reference; q needs no
        // normaliser (it is renormalised over the support)
        const float T = sp.temperature[row];
        inv_temp = 1.0 / static_cast<double>(T);
        const float Td = sp.draft_temperature ? sp.draft_temperature[row] : T;
        inv_temp_q = 1.0 / static_cast<double>(Td);
        if (!(Td > 0.f) || !(Td <= 3.0e38f)) bad = 1;
        float m = -__builtin_inff();
        for (int s = 0; s < sp.splits; ++s) m = fmaxf(m, sp.part_pref[row * sp.splits + s]);
        p_ref = static_cast<double>(m);
        for (int s = 0; s < sp.splits; ++s) {
            total += sp.cand_count[row * sp.splits + s];
            bad |= sp.part_bad[row * sp.splits + s];
            const float r = sp.part_pref[row * sp.splits + s];
            if (r > -3.0e38f) ptot += sp.part_psum[row * sp.splits + s] * exp((static_cast<double>(r) - p_ref) * inv_temp);
        }
        qtot = 1.0;
        if (!(ptot > 0.0) || !(ptot < 1e300) || !(m > -3.0e38f)) bad = 1;
    } else {
        for (int s = 0; s < sp.splits; ++s) {
            total += sp.cand_count[row * sp.splits + s];
            bad |= sp.part_bad[row * sp.splits + s];
            ptot += sp.part_psum[row * sp.splits + s];
            qtot += sp.part_qsum[row * sp.splits + s];
        }
        if (!(fabs(ptot - 1.0) <= 1e-3) || !(fabs(qtot - 1.0) <= 1e-3)) bad = 1;
    }
    info.p_total = ptot; info.q_total = qtot; info.p_ref = p_ref; info.inv_temp = sp.logits ? inv_temp : 0.0;
    if (bad || total <= 0 || total > kSelCap) {
        if (tid == 0) {
            info.status = GR_ROW_BAD;
            info.alpha_star = __longlong_as_double(0x7ff8000000000000ll);
            sp.info[row] = info;
            sp.accept_prob[row] = __uint_as_float(0x7fc00000u);
            sp.status[row] = GR_ROW_BAD;
            if (sp.v_drafts) { sp.v_token[row] = -1; sp.v_accepted[row] = 0; }
        }
        return;
    }
    {
        int off = 0;
        for (int s = 0; s < sp.splits; ++s) {
            const int c = sp.cand_count[row * sp.splits + s];
            const unsigned long long* src = sp.cand + (static_cast<size_t>(row) * sp.splits + s) * kMaxSupport;
            for (int i = tid; i < c; i += kST) L.keys[off + i] = src[i];
            off += c;
        }
    }
    if (tid == 0) { L.count = 0; L.work = 0.0; }
#ifdef GR_PHASE_CLOCKS
    if (tid == 0) { for (int i = 0; i < 24; ++i) L.clk[i] = 0; L.clk_last = clock64(); }
#endif
    __syncthreads();
    unsigned long long theta = 0ull;
    if (total > sp.k) theta = block_kth_largest<kST>(L.keys, total, sp.k, L.hist, L.pick);
    int kk = min(total, sp.k);
    for (int i = tid; i < total; i += kST) {
        const unsigned long long key = L.keys[i];
        if (key >= theta) {
            const int slot = atomicAdd(&L.count, 1);
            if (slot < KS) { L.ids[slot] = key_id(key); L.accb[slot] = static_cast<double>(sp.logits ? key_logit(key) : key_q(key)); }
        }
    }
    __syncthreads();
    if (sp.tail_mass > 0.0 && !sp.logits) {
        // Nucleus cut of the draft (Sec. 5.1: top-p/k sampling of the draft restricts the domain): the candidates by
        // decreasing q (ties by token id), their running sum added one after the other, and the support ends with the
        // first token at which it reaches (1 - tail_mass) of the row's q mass.
        int qr_ = 0;
        if (tid < kk) {
            const double qa = L.accb[tid]; const int ta = L.ids[tid];
            for (int j = 0; j < kk; ++j) { const double qj = L.accb[j]; qr_ += static_cast<int>(qj > qa) | (static_cast<int>(qj == qa) & static_cast<int>(L.ids[j] < ta)); }
            L.qd[qr_] = qa;
        }
        __syncthreads();
        {
#pragma clang fp contract(off)
            if ((tid >> 6) == 0) wave_sequential_scan(L.qd, L.S, kk, 0.0);
        }
        __syncthreads();
        const double need = (1.0 - sp.tail_mass) * qtot;
        const double first = block_min<kSW>((tid < kk && L.S[tid + 1] >= need) ? static_cast<double>(tid + 1) : static_cast<double>(kk), L.redn);
        const int keep = static_cast<int>(first);             // ranks 0 .. keep - 1 by q stay
        const bool stay = tid < kk && qr_ < keep;
        const int myid = tid < kk ? L.ids[tid] : 0; const double myq = tid < kk ? L.accb[tid] : 0.0;
        __syncthreads();
        if (stay) { L.ids[qr_] = myid; L.accb[qr_] = myq; }    // any order serves: the ranks are counted again below
        kk = keep;
        __syncthreads();
    }
    // unsorted: token ids in ids, q in accb (exact float values), p gathered into G0
    if (sp.logits) {
        // p = exp((t - p_ref) / T) (divided by the row's sum with the other p below), q = exp((d - largest d) / T),
        // and the two keys every order is decided on: d - t for the ratio (q/p is proportional to
        // exp((d - t) / T); exact for float32 logits) and d itself for q
        const double d = tid < kk ? L.accb[tid] : -1e300;
        const double dmax = block_max<kSW>(d, L.redn);
        if (tid < kk) {
            const double t = static_cast<double>(sp.p[static_cast<size_t>(row) * V + L.ids[tid]]);
            L.G0[tid] = exp((t - p_ref) * inv_temp);
            L.dlt[tid] = logit_ratio_key(d, t, inv_temp_q, inv_temp); L.dval[tid] = d;
            L.accb[tid] = exp((d - dmax) * inv_temp_q);
        }
    } else if (tid < kk) L.G0[tid] = static_cast<double>(sp.p[static_cast<size_t>(row) * V + L.ids[tid]]);
    if (tid < kk) { L.cnt0[tid] = 0; L.cnt1[tid] = 0; }
    __syncthreads();
    GR_CLK(L, 0);
    // ---- two orders from one pass of rank counting (`parts` threads share a token, each counts over a stretch
    // of the others): by decreasing q/p -- exact cross products (float x float fits a double), ties by id --
    // and by decreasing q, ties by id (the order in which truncation sets grow).
    {
        const int parts = kk <= kST / 4 ? 4 : (kk <= kST / 2 ? 2 : 1);
        const int per = kST / parts;                       // tokens a part can hold
        const int me = tid % per, part = tid / per;
        if (me < kk) {
            const int ta = L.ids[me];
            const int j0 = (kk * part) / parts, j1 = (kk * (part + 1)) / parts;
            int rank = 0, qrank = 0;
            if (sp.logits) {
                const double ka = L.dlt[me], da = L.dval[me];
#pragma unroll 4
                for (int j = j0; j < j1; ++j) {
                    const double kj = L.dlt[j], dj = L.dval[j];
                    const int lower = static_cast<int>(L.ids[j] < ta);
                    rank += static_cast<int>(kj > ka) | (static_cast<int>(kj == ka) & lower);
                    qrank += static_cast<int>(dj > da) | (static_cast<int>(dj == da) & lower);
                }
            } else {
                const double qa = L.accb[me], pa = L.G0[me];
#pragma unroll 4
                for (int j = j0; j < j1; ++j) {
                    const double qj = L.accb[j];
                    const double lhs = qj * pa, rhs = qa * L.G0[j];   // j before me?
                    const int lower = static_cast<int>(L.ids[j] < ta);
                    rank += static_cast<int>(lhs > rhs) | (static_cast<int>(lhs == rhs) & lower);
                    qrank += static_cast<int>(qj > qa) | (static_cast<int>(qj == qa) & lower);
                }
            }
            if (parts > 1) { atomicAdd(&L.cnt0[me], rank); atomicAdd(&L.cnt1[me], qrank); }
            else { L.cnt0[me] = rank; L.cnt1[me] = qrank; }
        }
        __syncthreads();
        if (tid < kk) {
            const int rank = L.cnt0[tid];
            L.tok[rank] = L.ids[tid]; L.qd[rank] = L.accb[tid]; L.pn[rank] = L.G0[tid] / ptot;
            L.byq[L.cnt1[tid]] = rank;                    // the token of q rank j sits at ratio rank byq[j]
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
    // ---- one wave, no barriers: H* (the smallest minimising prefix), the suffix minima G of F, residuals,
    // targets and records (F(m) <= G(m+1) for m >= h; m = kk always), the block of every token, and the
    // order by decreasing q split into H* and the rest.  Lane l holds ranks 5l .. 5l+4 (kk + 1 <= 257).
    if ((tid >> 6) == 0) {
        constexpr int E = (KS + 1 + 63) / 64;
        const int lane = tid, m0 = lane * E;
        double Fv[E];
#pragma unroll
        for (int e = 0; e < E; ++e) Fv[e] = (m0 + e <= kk) ? L.F[m0 + e] : 1e300;
        double lmin = Fv[0];
#pragma unroll
        for (int e = 1; e < E; ++e) lmin = fmin(lmin, Fv[e]);
        const double Fmin = wave_min(lmin);
        int lidx = 1 << 20;
#pragma unroll
        for (int e = E - 1; e >= 0; --e) if (Fv[e] == Fmin) lidx = m0 + e;
        const int hh = static_cast<int>(wave_min(static_cast<double>(lidx)));
        double sfx[E];
        sfx[E - 1] = Fv[E - 1];
#pragma unroll
        for (int e = E - 2; e >= 0; --e) sfx[e] = fmin(Fv[e], sfx[e + 1]);
        double later = sfx[0];                             // min of F over this lane's ranks and all later ones
        for (int o = 1; o < 64; o <<= 1) { const double x = __shfl_down(later, o); if (lane + o < 64) later = fmin(later, x); }
        double after = __shfl_down(later, 1);              // ... over the later lanes only
        if (lane == 63) after = 1e300;
        int fl[E], run = 0, cl[E];
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const int m = m0 + e;
            fl[e] = 0;
            if (m <= kk) {
                const double g = fmin(sfx[e], after);                                   // G(m)
                const double gn = (e < E - 1) ? fmin(sfx[e + 1], after) : after;         // G(m + 1), unused at m = kk
                fl[e] = (m >= hh && (m == kk || Fv[e] <= gn)) ? 1 : 0;
                L.flag[m] = fl[e];
                if (m < kk) {
                    const double r = (m >= hh) ? gn - g : 0.0;
                    L.rho[m] = r; L.tgt[m] = L.pn[m] - r;
                }
            }
            run += fl[e]; cl[e] = run;
        }
        int incl = run;
        for (int o = 1; o < 64; o <<= 1) { const int up = __shfl_up(incl, o); if (lane >= o) incl += up; }
        const int base = incl - run;
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const int m = m0 + e;
            if (m <= kk) {
                const int c = base + cl[e];
                if (fl[e]) L.blo[c] = m;                     // record number c (1-based) sits at rank m
                if (m < kk) L.blk[m] = (m >= hh) ? c : 0;    // token m (rank m+1) lies after record c
            }
        }
        const int nrec_ = __shfl(incl, 63);
        // ordq: ratio ranks listed by decreasing q, the tokens of H* first (a stable split of the q order)
        constexpr int E4 = KS / 64;
        const int j0 = lane * E4;
        int rk[E4], in[E4], cin = 0, ci[E4];
#pragma unroll
        for (int e = 0; e < E4; ++e) {
            const int j = j0 + e;
            rk[e] = j < kk ? L.byq[j] : 0;
            in[e] = (j < kk && rk[e] < hh) ? 1 : 0;
            ci[e] = cin;                                   // members of H* among this lane's earlier entries
            cin += in[e];
        }
        int incl_in = cin;
        for (int o = 1; o < 64; o <<= 1) { const int up = __shfl_up(incl_in, o); if (lane >= o) incl_in += up; }
        const int base_in = incl_in - cin;
#pragma unroll
        for (int e = 0; e < E4; ++e) {
            const int j = j0 + e;
            if (j < kk) {
                const int before_in = base_in + ci[e];
                L.ordq[in[e] ? before_in : hh + (j - before_in)] = rk[e];
            }
        }
        if (lane == 0) { L.pick[0] = hh; L.pick[1] = nrec_; }
    }
    __syncthreads();
    const int h = L.pick[0];
    const int nrec = L.pick[1];
    const int nblk = nrec - 1;
    GR_CLK(L, 2);
    // ---- truncation sets: fewest tokens by decreasing q with gamma_T <= tau / epsilon_T <= tau
    const double Qh = L.Q[h];
    {
#pragma clang fp contract(off)
        // running q mass in decreasing-q order: G0 <- q in that order, G1 <- its sequential prefix sums
        if (tid < kk) L.G0[tid] = L.qn[L.ordq[tid]];
        __syncthreads();
        if ((tid >> 6) == 0) wave_sequential_scan(L.G0, L.G1, h, 0.0);
        if ((tid >> 6) == 1) wave_sequential_scan(L.G0 + h, L.G1 + h + 1, kk - h, Qh);
        __syncthreads();
        // the token at position t of that order has the mass G1[...] before it
        if (tid < kk) {
            const int j = L.ordq[tid];
            const double a = L.G1[tid < h ? tid : tid + 1];
            const double an = (a > 0.0) ? ipow(a, n) : 0.0;
            L.inT[j] = (j < h) ? ((ipow(Qh, n) - an) > sp.tau) : ((1.0 - an) > sp.tau);
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
    int status = GR_ROW_OK, evals = 0, par = 0;
    for (int b = (h > 0 ? 0 : 1); b <= nblk && status != GR_ROW_TRUNC_CAP; ++b) {
        const int lo = (b == 0) ? 0 : L.blo[b];
        const int hi = (b == 0) ? h : L.blo[b + 1];
        if (b > 0 && hi - lo < 2) continue;
        const int m = compact_active(L, lo, hi, kk);
        if (m > sp.max_T) { status = GR_ROW_TRUNC_CAP; break; }
        if (m == 0 || (b > 0 && m < 2)) continue;
        double w0 = 0.0, q0 = 0.0, t0 = 0.0;
        if (tid < m) {
            const int j = L.apos[tid];
            w0 = L.wgt[j]; q0 = L.qn[j]; t0 = L.tgt[j];
            L.aq[tid] = q0; L.aal[tid] = fast_log(w0);
        }
        // one exchange: the draw mass and the targets of the active tokens, their start weights, and (inner
        // system) the context = tokens of T with target 0 (weight 0): they fill tuples but take no mass
        double ex[4] = {wave_sum(q0), wave_sum(t0), wave_sum(w0),
                        wave_sum((b == 0 && tid < h && L.inT[tid] && !(L.tgt[tid] > 0.0)) ? L.qn[tid] : 0.0)};
        wg_reduce<4>(L, par, ex, {kOpSum, kOpSum, kOpSum, kOpSum});
        const double qa = ex[0], ta = ex[1], w0sum = ex[2];
        double ctx, scale, slack_target = 0.0;
        if (b == 0) {
            ctx = ex[3];
            const double mass = ipow(ctx + qa, n);
            scale = mass / (ta - L.F[h]);
            slack_target = -L.F[h] * scale;
        } else {
            ctx = L.Q[lo];
            scale = pow_diff(ctx + qa, qa, n) / ta;
        }
        if (tid < m) L.at[tid] = t0 * scale;
        GR_CLK(L, 4);
        const int rc = solve_program<D>(L, par, sp.newton_ws + static_cast<size_t>(row) * kMaxT * (kMaxT + 1), m, n, ctx, b == 0, slack_target,
                                        qa, ta * scale, sp.rel_tol, sp.max_iter, &evals);
        if (rc != 0 && status == GR_ROW_OK) status = GR_ROW_ITER_CAP;
        const double wv = (tid < m) ? exp(L.aal[tid]) : 0.0;
        const double wsum = (b == 0) ? 1.0 : wg_sum(L, par, wv);
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
    info.support = kk; info.h = h; info.status = status; info.iterations = evals;
    info.alpha_star = 1.0 + L.F[h];
    info.res_total = -L.F[h];
    info.node_tokens = L.work;
    if (tid == 0) {
#ifdef GR_PHASE_CLOCKS
        { const long long now_ = clock64(); L.clk[14] += now_ - L.clk_last; for (int i = 0; i < 24; ++i) { info.clk[i] = L.clk[i]; info.errlog[i] = i < evals ? L.errlog[i] : 0.0; } }
#endif
        sp.info[row] = info;
        sp.accept_prob[row] = static_cast<float>(1.0 + L.F[h]);
        sp.status[row] = status;
    }
    // ---- the row's verification, when the drafts came with the call: the same routine as verify_kernel, run by the
    // first kThreads threads on the policy this workgroup has just written (visible to it behind the barrier).  The
    // other waves end here; a workgroup barrier waits for the waves that are still alive only.
    if (sp.v_drafts) {
        __syncthreads();
        if (tid >= kThreads) __builtin_amdgcn_endpgm();
        RowPolicy rp;
        rp.o = o_order; rp.bl = o_block; rp.wt = o_w; rp.rh = o_rho; rp.rk = nullptr; rp.rid = nullptr;
        rp.pieces = sp.piece_psum ? sp.piece_psum + static_cast<size_t>(row) * sp.piece_stride : nullptr;
        rp.prefs = sp.piece_pref ? sp.piece_pref + static_cast<size_t>(row) * sp.piece_stride : nullptr;
        static_assert(sizeof(VerifyLds) <= sizeof(Lds<D>), "the verification reuses the solve's LDS");
        verify_row(*reinterpret_cast<VerifyLds*>(gr_lds_raw), sp.p + static_cast<size_t>(row) * sp.V, sp.V, sp.n, rp, info,
                   sp.v_drafts + static_cast<size_t>(row) * sp.n, sp.v_uniforms[row], sp.v_token + row, sp.v_accepted + row);
    }
}

// ---- full-vocabulary policies: the convex programs of a row whose steps 1-2 were done in HBM.
// Start weights of every support token, the dense per-token arrays the verify kernel reads, then the
// inner program over T inside H* and one outer program per block that holds two or more active
// tokens of T -- the same programs, in the same arithmetic, as the LDS-resident path.
template <int D>
__global__ __launch_bounds__(kThreadsOf<D>) void full_programs_kernel(FullParams fp) {
    constexpr int kST = Lds<D>::kST, kSW = Lds<D>::kSW;
    Lds<D>& L = *reinterpret_cast<Lds<D>*>(gr_lds_raw);
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

    // a row that exceeded the cap on |T| is sampled from p (no dense arrays, no weights are read for it)
    if (info.status != GR_ROW_OK) return;
    // tokens outside the support keep all of p as residual; then the support by rank
    if (fp.logits) {
        for (int i = tid; i < V; i += kST) { rank_of[i] = -1; rho_id[i] = exp((static_cast<double>(pr[i]) - info.p_ref) * info.inv_temp) / info.p_total; }
    } else {
        for (int i = tid; i < V; i += kST) { rank_of[i] = -1; rho_id[i] = static_cast<double>(pr[i]) / info.p_total; }
    }
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

    int status = GR_ROW_OK, evals = 0, par = 0;
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
        const double ctx = block_sum<kSW>(ctx_part, L.redn);
        if (m > 0 && m <= kMaxT) {
            const double qa = block_sum<kSW>(tid < m ? L.aq[tid] : 0.0, L.redn);
            const double ta = block_sum<kSW>(tid < m ? L.at[tid] : 0.0, L.redn);
            const double mass = ipow(ctx + qa, n);
            const double scale = mass / (ta - Fh);
            const double slack_target = -Fh * scale;
            if (tid < m) L.at[tid] *= scale;
            __syncthreads();
            const int rc = solve_program<D>(L, par, fp.newton_ws + static_cast<size_t>(row) * kMaxT * (kMaxT + 1), m, n, ctx, 1, slack_target,
                                            qa, ta * scale, fp.rel_tol, fp.max_iter, &evals);
            if (rc != 0) status = GR_ROW_ITER_CAP;
            if (tid < m) weight[L.apos[tid]] = exp(L.aal[tid]);
            __syncthreads();
        }
    }
    // ---- outer programs: those blocks with two or more active tokens of T
    const int nblk = fp.nblk[row];
    for (int b0 = 1; b0 <= nblk; b0 += KS) {               // windows of KS blocks: L.flag lists the window's programs
        const int bme = b0 + tid;
        const bool need = tid < KS && bme <= nblk && bcount[bme] >= 2;
        const unsigned long long nmask = __ballot(need);
        if (lane == 0) L.hist[wv] = __popcll(nmask);
        __syncthreads();
        int pslot = __popcll(nmask & ((1ull << lane) - 1ull));
        int nprog = 0;
        for (int w = 0; w < kSW; ++w) { if (w < wv) pslot += L.hist[w]; nprog += L.hist[w]; }
        if (need) L.flag[pslot] = bme;                      // nprog <= KS
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
            const double qa = block_sum<kSW>(tid < m ? L.aq[tid] : 0.0, L.redn);
            const double ta = block_sum<kSW>(tid < m ? L.at[tid] : 0.0, L.redn);
            const double ctx = Q[lo];
            const double scale = pow_diff(ctx + qa, qa, n) / ta;
            const double w0sum = block_sum<kSW>(tid < m ? exp(L.aal[tid]) : 0.0, L.redn);
            if (tid < m) L.at[tid] *= scale;
            __syncthreads();
            const int rc = solve_program<D>(L, par, fp.newton_ws + static_cast<size_t>(row) * kMaxT * (kMaxT + 1), m, n, ctx, 0, 0.0,
                                            qa, ta * scale, fp.rel_tol, fp.max_iter, &evals);
            if (rc != 0 && status == GR_ROW_OK) status = GR_ROW_ITER_CAP;
            const double wvv = (tid < m) ? exp(L.aal[tid]) : 0.0;
            const double wsum = block_sum<kSW>(wvv, L.redn);
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
    const dim3 grid(fp.B);
    if (fp.n <= 2) hipLaunchKernelGGL(full_programs_kernel<2>, grid, dim3(kThreadsOf<2>), sizeof(Lds<2>), stream, fp);
    else if (fp.n <= 4) hipLaunchKernelGGL(full_programs_kernel<4>, grid, dim3(kThreadsOf<4>), sizeof(Lds<4>), stream, fp);
    else if (fp.n <= 8) hipLaunchKernelGGL(full_programs_kernel<8>, grid, dim3(kThreadsOf<8>), sizeof(Lds<8>), stream, fp);
    else hipLaunchKernelGGL(full_programs_kernel<16>, grid, dim3(kThreadsOf<16>), sizeof(Lds<16>), stream, fp);
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
    const dim3 grid(sp.B);
    if (sp.n <= 2) hipLaunchKernelGGL(solve_kernel<2>, grid, dim3(kThreadsOf<2>), sizeof(Lds<2>), stream, sp);
    else if (sp.n <= 4) hipLaunchKernelGGL(solve_kernel<4>, grid, dim3(kThreadsOf<4>), sizeof(Lds<4>), stream, sp);
    else if (sp.n <= 8) hipLaunchKernelGGL(solve_kernel<8>, grid, dim3(kThreadsOf<8>), sizeof(Lds<8>), stream, sp);
    else hipLaunchKernelGGL(solve_kernel<16>, grid, dim3(kThreadsOf<16>), sizeof(Lds<16>), stream, sp);
    return hipGetLastError();
}

}  // namespace gr
