// Per-row solve: one 256-thread workgroup per decode position, everything after the streaming
// selection lives in LDS.
//
//   merge the slices' candidates -> top-k support V_0       (App. "Top-k Sampling ...")
//   order by decreasing q/p, prefix psi, H*, alpha*         (Sec. 5.1, Thm 3.1)
//   suffix minima -> outer targets p_i and block boundaries (Thm 6.2, Lemma 6.3)
//   truncation sets T                                       (Alg. 1, Sec. 6.3)
//   softmax weights of Theta_T / Phi_T by iterative scaling (Thm 6.5 / Thm 6.4)
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

constexpr int KS = kMaxSupport;
constexpr double kQuadStep = 0.45;   // trapezoid step in log t (discretisation error ~1e-8 relative)
constexpr double kQuadLo = 1e-4;     // t_lo * (slack + sum w): the part below t_lo is added in closed form
constexpr double kQuadHi = 25.0;     // t_hi * (slowest decay rate)
constexpr int kCols = kHist - 1;                       // Anderson columns
constexpr int kGram = kCols * (kCols + 1) / 2 + kCols; // upper triangle of the Gram matrix + right-hand side

struct Lds {
    // support, in ratio order
    int tok[KS]; int blk[KS]; int inT[KS]; int ordq[KS]; int apos[kMaxT];
    int flag[KS + 2]; int cnt0[KS + 2]; int cnt1[KS + 2]; int blo[KS + 2];
    double qd[KS]; double qn[KS]; double pn[KS]; double rho[KS]; double tgt[KS]; double wgt[KS]; double accb[KS];
    double P[KS + 1]; double S[KS + 1]; double Q[KS + 1]; double F[KS + 2]; double G0[KS + 2]; double G1[KS + 2];
    // one convex program
    double aq[kMaxT]; double at[kMaxT]; double aal[kMaxT]; double aw[kMaxT]; double aR[kMaxT]; double af[kMaxT];
    double Ha[kHist][kMaxT]; double Hf[kHist][kMaxT]; double aBest[kMaxT]; double fBest[kMaxT];
    double gram[kWaves][kGram]; double gamma[kCols];
    double red[kWaves]; double R0acc; int ok; int pick[2]; int count; int hist[256];
    // unsorted candidates (select merge), later the per-wave partial products of the evaluator
    union {
        unsigned long long keys[kSelCap];
        double part[kWaves * 17 * 64];
    } u;
};

#pragma clang fp contract(off)
__device__ __forceinline__ double ipow(double x, int n) {
    double r = x;
    for (int i = 1; i < n; ++i) r = r * x;
    return r;
}

// a^n - (a-d)^n without cancellation
__device__ __forceinline__ double pow_diff(double a, double d, int n) {
    const double b = a - d;
    double ap[GR_MAX_N], bp[GR_MAX_N];
    ap[0] = 1.0; bp[0] = 1.0;
    for (int i = 1; i < n; ++i) { ap[i] = ap[i - 1] * a; bp[i] = bp[i - 1] * b; }
    double s = 0.0;
    for (int i = 0; i < n; ++i) s = s + ap[n - 1 - i] * bp[i];
    return d * s;
}
#pragma clang fp contract(fast)

// Routed mass of every active token, and the mass left to the slack term.
// In: L.aq (q of the active tokens), L.aal (log weights), m, n, ctx, slack, qsum = sum aq.
// Out: L.aR[0..m), L.R0acc (slack mass; meaningful when slack = 1).  All threads call it.
template <int D>
__device__ void routed_eval(Lds& L, int m, int n, double ctx, int slack, double qsum, int* nodes_used) {
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    double w = 0.0;
    if (tid < m) { w = exp(L.aal[tid]); L.aw[tid] = w; }
    const double wsum = block_sum(tid < m ? w : 0.0, L.red);
    const double wmin = block_min(tid < m ? w : 1e300, L.red);
    const double t_lo = kQuadLo / (slack + wsum);
    const double t_hi = kQuadHi / (slack + ((slack == 0 || ctx == 0.0) ? wmin : 0.0));
    const double range = log(t_hi / t_lo);
    double step = kQuadStep;
    int N = static_cast<int>(ceil(range / step)) + 1;
    if (N > 64 && range <= 0.5 * 63.0) { step = range / 63.0; N = 64; }
    if (N < 1) N = 1;
    if (N > 4096) N = 4096;
    *nodes_used = N;
    const double atot = ctx + qsum;
    const double tail = step * t_lo / (exp(step) - 1.0);   // trapezoid sum of the nodes below t_lo, x = 1 there
    double fact = 1.0;
    for (int i = 2; i <= n; ++i) fact *= i;
    if (tid < m) L.aR[tid] = pow_diff(atot, L.aq[tid], n) * tail / fact;
    if (tid == 0) L.R0acc = ipow(atot, n) * tail / fact;
    __syncthreads();

    for (int c0 = 0; c0 < N; c0 += 64) {
        const int node = c0 + lane;
        const double t = t_lo * exp(step * node);
        const double qw = node < N ? step * t * exp(-slack * t) : 0.0;
        // phase 1: this wave's partial product over its tokens
        double A[D + 1];
        A[0] = 1.0;
#pragma unroll
        for (int d = 1; d <= D; ++d) A[d] = 0.0;
        for (int i = wv; i < m; i += kWaves) {
            const double x = exp(-t * L.aw[i]);
            const double q = L.aq[i];
            double e[D + 1];
            e[0] = 1.0;
#pragma unroll
            for (int a = 1; a <= D; ++a) e[a] = e[a - 1] * q / a;
#pragma unroll
            for (int d = D; d >= 1; --d) {
                double acc = 0.0;
#pragma unroll
                for (int a = 1; a <= d; ++a) acc = fma(e[a], A[d - a], acc);
                A[d] = fma(x, acc, A[d]);
            }
        }
#pragma unroll
        for (int d = 0; d <= D; ++d) L.u.part[(wv * (D + 1) + d) * 64 + lane] = A[d];
        __syncthreads();
        // phase 2: total product, context included
        double T[D + 1];
        T[0] = 1.0;
#pragma unroll
        for (int d = 1; d <= D; ++d) T[d] = T[d - 1] * ctx / d;
        for (int w2 = 0; w2 < kWaves; ++w2) {
            double Bc[D + 1];
#pragma unroll
            for (int d = 0; d <= D; ++d) Bc[d] = L.u.part[(w2 * (D + 1) + d) * 64 + lane];
#pragma unroll
            for (int d = D; d >= 0; --d) {
                double acc = 0.0;
#pragma unroll
                for (int a = 0; a <= d; ++a) acc = fma(T[a], Bc[d - a], acc);
                T[d] = acc;
            }
        }
        // phase 3: leave one token out by series division, take the z^n coefficient
        for (int i = wv; i < m; i += kWaves) {
            const double x = exp(-t * L.aw[i]);
            const double q = L.aq[i];
            double e[D + 1];
            e[0] = 1.0;
#pragma unroll
            for (int a = 1; a <= D; ++a) e[a] = e[a - 1] * q / a;
            double Bq[D + 1];
            Bq[0] = T[0];
            double cn = 0.0;
#pragma unroll
            for (int d = 1; d <= D; ++d) {
                double conv = 0.0;
#pragma unroll
                for (int a = 1; a <= d; ++a) conv = fma(e[a], Bq[d - a], conv);
                Bq[d] = fma(-x, conv, T[d]);
                if (d == n) cn = conv;
            }
            const double v = wave_sum(qw * x * cn);
            if (lane == 0) L.aR[i] += v;
        }
        if (wv == 0) {
            double tn = 0.0;
#pragma unroll
            for (int d = 0; d <= D; ++d) if (d == n) tn = T[d];
            const double v = wave_sum(qw * tn);
            if (lane == 0) L.R0acc += v;
        }
        __syncthreads();
    }
    if (tid < m) L.aR[tid] *= L.aw[tid] * fact;
    if (tid == 0) L.R0acc *= fact * slack;
    __syncthreads();
}

// Solve one program by iterative scaling with Anderson mixing.  Returns 0 when converged.
// In: L.aq, L.at (targets, already scaled to the tuple mass), L.aal (start log weights).
// Out: L.aal.  `evals` counts evaluator calls.
template <int D>
__device__ int solve_program(Lds& L, int m, int n, double ctx, int slack, double slack_target,
                             double rel_tol, int max_iter, int* evals) {
    const int tid = threadIdx.x;
    const double qsum = block_sum(tid < m ? L.aq[tid] : 0.0, L.red);
    const double tsum = block_sum(tid < m ? L.at[tid] : 0.0, L.red);
    int hcount = 0, plain = 0;
    double best_err = 1e300;
    int result = 1;
    for (int it = 1; it <= max_iter; ++it) {
        if (!slack) {
            const double amax = block_max(tid < m ? L.aal[tid] : -1e300, L.red);
            if (tid < m) L.aal[tid] -= amax;
            __syncthreads();
        }
        int nodes;
        routed_eval<D>(L, m, n, ctx, slack, qsum, &nodes);
        *evals += 1;
        // Without slack the routed masses sum to the tuple mass identically, so only the ratios
        // R_i / target_i carry information; dividing by their common value also removes the
        // (common) relative error of the quadrature from the stopping test.
        const double rsum = slack ? 0.0 : block_sum(tid < m ? L.aR[tid] : 0.0, L.red);
        double f = 0.0;
        if (tid < m) {
            f = log(L.at[tid] / L.aR[tid]);
            f -= slack ? log(slack_target / L.R0acc) : log(tsum / rsum);
            L.af[tid] = f;
        }
        const double err = block_max(tid < m ? fabs(f) : 0.0, L.red);
#ifdef GR_DEBUG
        if (tid == 0 && blockIdx.x == GR_DEBUG) printf("it %d m %d slack %d err %.3e nodes %d a0 %.6f a1 %.6f R0 %.6e R1 %.6e t0 %.6e t1 %.6e R0acc %.3e hcount %d\n", it, m, slack, err, nodes, L.aal[0], L.aal[1], L.aR[0], L.aR[1], L.at[0], L.at[1], L.R0acc, hcount);
#endif
        if (err <= rel_tol) { result = 0; break; }
        if (!(err < 1e300) || err > 100.0 * best_err) {
            // a mixed step went astray: back to the best point, plain (monotone) steps for a while
            if (!(best_err < 1e300)) break;        // no finite point seen: give up on this program
            if (tid < m) { L.aal[tid] = L.aBest[tid]; f = L.fBest[tid]; }
            hcount = 0; plain = 20;
        } else if (err < best_err) {
            best_err = err;
            if (tid < m) { L.aBest[tid] = L.aal[tid]; L.fBest[tid] = f; }
        }
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
            double prod[kGram];
            int e = 0;
#pragma unroll
            for (int a = 0; a < kCols; ++a)
#pragma unroll
                for (int b = a; b < kCols; ++b) prod[e++] = dF[a] * dF[b];
#pragma unroll
            for (int a = 0; a < kCols; ++a) prod[e++] = dF[a] * f;
#pragma unroll
            for (int j = 0; j < kGram; ++j) {
                const double s = wave_sum(prod[j]);
                if ((tid & 63) == 0) L.gram[tid >> 6][j] = s;
            }
            __syncthreads();
            if (tid == 0) {
                double Gm[kCols][kCols + 1];
                int idx = 0;
                for (int a = 0; a < kCols; ++a)
                    for (int b = a; b < kCols; ++b) {
                        const double g = L.gram[0][idx] + L.gram[1][idx] + L.gram[2][idx] + L.gram[3][idx];
                        Gm[a][b] = g; Gm[b][a] = g; ++idx;
                    }
                double tr = 0.0;
                for (int a = 0; a < ncol; ++a) tr += Gm[a][a];
                for (int a = 0; a < kCols; ++a) {
                    Gm[a][kCols] = L.gram[0][idx] + L.gram[1][idx] + L.gram[2][idx] + L.gram[3][idx]; ++idx;
                    Gm[a][a] += 1e-13 * tr + 1e-300;
                }
                int good = 1;
                for (int c = 0; c < ncol && good; ++c) {            // Gaussian elimination, partial pivoting
                    int piv = c;
                    for (int r = c + 1; r < ncol; ++r) if (fabs(Gm[r][c]) > fabs(Gm[piv][c])) piv = r;
                    if (!(fabs(Gm[piv][c]) > 0.0)) { good = 0; break; }
                    if (piv != c) for (int j = 0; j <= kCols; ++j) { double tmp = Gm[c][j]; Gm[c][j] = Gm[piv][j]; Gm[piv][j] = tmp; }
                    for (int r = c + 1; r < ncol; ++r) {
                        const double fct = Gm[r][c] / Gm[c][c];
                        for (int j = c; j <= kCols; ++j) Gm[r][j] -= fct * Gm[c][j];
                    }
                }
                if (good) {
                    for (int c = ncol - 1; c >= 0; --c) {
                        double s = Gm[c][kCols];
                        for (int j = c + 1; j < ncol; ++j) s -= Gm[c][j] * L.gamma[j];
                        L.gamma[c] = s / Gm[c][c];
                    }
                }
                for (int c = ncol; c < kCols; ++c) L.gamma[c] = 0.0;
                L.ok = good;
            }
            __syncthreads();
            double cand = f;
#pragma unroll
            for (int c = 0; c < kCols; ++c) cand -= (dA[c] + dF[c]) * L.gamma[c];
            const int solved = L.ok;
            const double cmax = block_max(tid < m ? fabs(cand) : 0.0, L.red);
            if (solved && cmax <= 10.0 * fmax(1.0, fmin(err, best_err))) stepv = cand;
            else hcount = 0;
        }
        if (tid < m) L.aal[tid] += stepv;
        ++hcount;
        __syncthreads();
    }
    __syncthreads();
    return result;
}

__device__ int dispatch_solve(Lds& L, int m, int n, double ctx, int slack, double slack_target,
                              double rel_tol, int max_iter, int* evals) {
    if (n <= 2) return solve_program<2>(L, m, n, ctx, slack, slack_target, rel_tol, max_iter, evals);
    if (n <= 4) return solve_program<4>(L, m, n, ctx, slack, slack_target, rel_tol, max_iter, evals);
    if (n <= 8) return solve_program<8>(L, m, n, ctx, slack, slack_target, rel_tol, max_iter, evals);
    return solve_program<16>(L, m, n, ctx, slack, slack_target, rel_tol, max_iter, evals);
}

// Build the active list of one program from a predicate over support positions [lo, hi), in
// ascending position.  Returns m (possibly > kMaxT, in which case nothing was written beyond kMaxT).
__device__ int compact_active(Lds& L, int lo, int hi) {
    const int tid = threadIdx.x;
    const int j = lo + tid;                              // hi - lo <= KS = kThreads
    const int on = (j < hi && L.inT[j] && L.tgt[j] > 0.0) ? 1 : 0;
    // inclusive scan of `on` over the workgroup
    int incl = on;
    for (int o = 1; o < 64; o <<= 1) { const int up = __shfl_up(incl, o); if ((tid & 63) >= o) incl += up; }
    int* wtot = reinterpret_cast<int*>(L.red);
    if ((tid & 63) == 63) wtot[tid >> 6] = incl;
    __syncthreads();
    int base = 0, total = 0;
    for (int w = 0; w < kWaves; ++w) { if (w < (tid >> 6)) base += wtot[w]; total += wtot[w]; }
    const int slot = base + incl - 1;
    if (on && slot < kMaxT) L.apos[slot] = j;
    __syncthreads();
    return total;
}

}  // namespace

__global__ __launch_bounds__(kThreads) void solve_kernel(SolveParams sp) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    Lds& L = *reinterpret_cast<Lds*>(lds_raw);
    const int tid = threadIdx.x;
    const int row = blockIdx.x;
    const int n = sp.n, V = sp.V;
    RowInfo info;
    info.support = 0; info.h = 0; info.status = GR_ROW_OK; info.iterations = 0;
    info.alpha_star = 0.0; info.res_total = 0.0; info.p_total = 0.0; info.q_total = 0.0;

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
            for (int i = tid; i < c; i += kThreads) L.u.keys[off + i] = src[i];
            off += c;
        }
    }
    if (tid == 0) L.count = 0;
    __syncthreads();
    unsigned long long theta = 0ull;
    if (total > sp.k) theta = block_kth_largest(L.u.keys, total, sp.k, L.hist, L.pick);
    const int kk = min(total, sp.k);
    for (int i = tid; i < total; i += kThreads) {
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

    // ---- order by decreasing q/p: exact cross products (float x float fits a double), ties by id
    if (tid < kk) {
        const double qa = L.accb[tid], pa = L.G0[tid];
        const int ta = L.ordq[tid];
        int rank = 0;
        for (int j = 0; j < kk; ++j) {
            const double lhs = L.accb[j] * pa, rhs = qa * L.G0[j];   // j before me?
            rank += (lhs > rhs) || (lhs == rhs && L.ordq[j] < ta);
        }
        L.tok[rank] = ta; L.qd[rank] = qa; L.pn[rank] = pa / ptot;
    }
    __syncthreads();

    // ---- prefix sums in the order, sequentially (bit-reproducible), then F(m) = P_m - Q_m^n
    {
#pragma clang fp contract(off)
        if (tid == 0) { double a = 0.0; L.P[0] = 0.0; for (int j = 0; j < kk; ++j) { a = a + L.pn[j]; L.P[j + 1] = a; } }
        if (tid == 64) { double a = 0.0; L.S[0] = 0.0; for (int j = 0; j < kk; ++j) { a = a + L.qd[j]; L.S[j + 1] = a; } }
        __syncthreads();
        const double stot = L.S[kk];
        for (int m = tid; m <= kk; m += kThreads) {
            const double Qm = L.S[m] / stot;
            L.Q[m] = Qm;
            L.F[m] = (m == 0) ? 0.0 : L.P[m] - ipow(Qm, n);
            if (m < kk) L.qn[m] = L.qd[m] / stot;
        }
        __syncthreads();
    }

    // ---- H*: the smallest minimising prefix
    double fmin_local = 1e300;
    for (int m = tid; m <= kk; m += kThreads) fmin_local = fmin(fmin_local, L.F[m]);
    const double Fmin = block_min(fmin_local, L.red);
    double hcand = 1e9;
    for (int m = tid; m <= kk; m += kThreads) if (L.F[m] == Fmin) hcand = fmin(hcand, static_cast<double>(m));
    const int h = static_cast<int>(block_min(hcand, L.red));

    // ---- G = suffix minima of F (Hillis-Steele over kk+1 entries)
    for (int m = tid; m <= kk; m += kThreads) L.G0[m] = L.F[m];
    __syncthreads();
    {
        double* src = L.G0; double* dst = L.G1;
        for (int o = 1; o <= kk; o <<= 1) {
            for (int m = tid; m <= kk; m += kThreads) dst[m] = (m + o <= kk) ? fmin(src[m], src[m + o]) : src[m];
            __syncthreads();
            double* t = src; src = dst; dst = t;
        }
        if (src != L.G0) { for (int m = tid; m <= kk; m += kThreads) L.G0[m] = src[m]; }
        __syncthreads();
    }
    // residuals, targets, records (F(m) <= G(m+1) for m >= h; m = kk always)
    for (int m = tid; m <= kk; m += kThreads) {
        L.flag[m] = (m >= h && (m == kk || L.F[m] <= L.G0[m + 1])) ? 1 : 0;
        if (m < kk) {
            const double r = (m >= h) ? L.G0[m + 1] - L.G0[m] : 0.0;
            L.rho[m] = r; L.tgt[m] = L.pn[m] - r;
        }
    }
    __syncthreads();
    // inclusive count of records -> block id of each token outside H*, and block bounds
    for (int m = tid; m <= kk; m += kThreads) L.cnt0[m] = L.flag[m];
    __syncthreads();
    {
        int* src = L.cnt0; int* dst = L.cnt1;
        for (int o = 1; o <= kk; o <<= 1) {
            for (int m = tid; m <= kk; m += kThreads) dst[m] = (m >= o) ? src[m] + src[m - o] : src[m];
            __syncthreads();
            int* t = src; src = dst; dst = t;
        }
        if (src != L.cnt0) { for (int m = tid; m <= kk; m += kThreads) L.cnt0[m] = src[m]; }
        __syncthreads();
    }
    const int nrec = L.cnt0[kk];
    const int nblk = nrec - 1;
    for (int m = tid; m <= kk; m += kThreads) {
        if (L.flag[m]) L.blo[L.cnt0[m]] = m;             // record number c (1-based) sits at rank m
        if (m < kk) L.blk[m] = (m >= h) ? L.cnt0[m] : 0; // token m (rank m+1) lies after record cnt0[m]
    }
    __syncthreads();

    // ---- truncation sets: fewest tokens by decreasing q with gamma_T <= tau / epsilon_T <= tau
    if (tid < kk) {
        const int mine_in = tid < h;
        const float qa = static_cast<float>(L.qd[tid]);
        const int ta = L.tok[tid];
        int rank = 0;
        for (int j = 0; j < kk; ++j) {
            const int same = (j < h) == mine_in;
            const float qj = static_cast<float>(L.qd[j]);
            rank += same && ((qj > qa) || (qj == qa && L.tok[j] < ta));
        }
        L.ordq[(mine_in ? 0 : h) + rank] = tid;
    }
    __syncthreads();
    const double Qh = L.Q[h];
    {
#pragma clang fp contract(off)
        if (tid == 0) { double a = 0.0; for (int r = 0; r < h; ++r) { const int j = L.ordq[r]; L.accb[j] = a; a = a + L.qn[j]; } }
        if (tid == 64) { double a = Qh; for (int r = h; r < kk; ++r) { const int j = L.ordq[r]; L.accb[j] = a; a = a + L.qn[j]; } }
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

    // ---- the convex programs: program 0 = inner system, then every outer block of two or more tokens
    int status = GR_ROW_OK, evals = 0;
    for (int b = (h > 0 ? 0 : 1); b <= nblk && status != GR_ROW_TRUNC_CAP; ++b) {
        const int lo = (b == 0) ? 0 : L.blo[b];
        const int hi = (b == 0) ? h : L.blo[b + 1];
        if (b > 0 && hi - lo < 2) continue;
        const int m = compact_active(L, lo, hi);
        if (m > sp.max_T) { status = GR_ROW_TRUNC_CAP; break; }
        if (m == 0 || (b > 0 && m < 2)) continue;
        if (tid < m) {
            const int j = L.apos[tid];
            L.aq[tid] = L.qn[j]; L.at[tid] = L.tgt[j]; L.aal[tid] = log(L.wgt[j]);
        }
        __syncthreads();
        const double qa = block_sum(tid < m ? L.aq[tid] : 0.0, L.red);
        const double ta = block_sum(tid < m ? L.at[tid] : 0.0, L.red);
        double ctx, scale, slack_target = 0.0;
        if (b == 0) {
            // context = tokens of T with target 0 (weight 0): they fill tuples but take no mass
            const int j = tid;
            ctx = block_sum((j < h && L.inT[j] && !(L.tgt[j] > 0.0)) ? L.qn[j] : 0.0, L.red);
            const double mass = ipow(ctx + qa, n);
            scale = mass / (ta - L.F[h]);
            slack_target = -L.F[h] * scale;
        } else {
            ctx = L.Q[lo];
            scale = pow_diff(ctx + qa, qa, n) / ta;
        }
        const double w0sum = block_sum(tid < m ? L.wgt[L.apos[tid]] : 0.0, L.red);
        if (tid < m) L.at[tid] *= scale;
        __syncthreads();
        const int rc = dispatch_solve(L, m, n, ctx, b == 0, slack_target, sp.rel_tol, sp.max_iter, &evals);
        if (rc != 0 && status == GR_ROW_OK) status = GR_ROW_ITER_CAP;
        const double wv = (tid < m) ? exp(L.aal[tid]) : 0.0;
        const double wsum = block_sum(wv, L.red);
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
        sp.info[row] = info;
        sp.accept_prob[row] = static_cast<float>(1.0 + L.F[h]);
        sp.status[row] = status;
    }
}

hipError_t solve_kernel_setup() {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(solve_kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(sizeof(Lds)));
}

hipError_t launch_solve(const SolveParams& sp, hipStream_t stream) {
    hipLaunchKernelGGL(solve_kernel, dim3(sp.B), dim3(kThreads), sizeof(Lds), stream, sp);
    return hipGetLastError();
}

}  // namespace gr
