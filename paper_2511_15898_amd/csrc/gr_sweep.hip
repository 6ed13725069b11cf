// Acceptance-only sweep: alpha*(k, n) = 1 + min_H psi(H) (Thm 3.1) for a grid of top-k sizes and numbers
// of i.i.d. drafts, per row, behind ONE streaming selection pass over p and q (with the largest k of
// the grid).  Sec. 5.1: the minimiser is a prefix of the order by decreasing q/p; for a smaller top-k
// the support is the first k tokens by decreasing q (App. "Top-k Sampling for the Relaxed OTLP") and
// its ratio order is the sub-sequence of the largest support's order, so one ordering serves the grid.
//
// One 256-thread workgroup per row, everything in LDS; thread m owns rank m of the ratio order.
// Only the minimum of F(m) = P_m - Q_m^n is reported, to 1e-5, so the prefix sums here are parallel
// scans in float64 (no integer decision hangs on their rounding).
#include <hip/hip_runtime.h>

#include "gr_internal.h"

namespace gr {

namespace {

struct SweepLds {
    unsigned long long keys[kSelCap];     // merged slice candidates
    unsigned long long ckey[kMaxSupport]; // the kmax largest, unordered
    double pv[kMaxSupport]; double qv[kMaxSupport];   // by slot
    double rp[kMaxSupport]; double rq[kMaxSupport];   // by ratio rank: p / sum p, raw q
    int rqr[kMaxSupport];                 // by ratio rank: the token's rank by decreasing q
    int ids[kMaxSupport];
    double wtot[2][kWaves];
    double cell[kSweepMaxN][kWaves];      // per draft count: the waves' minima of F
    int hist[256]; int pick[4]; int count;
};

// Inclusive sums of a and b over the 256 threads (thread order); *atot, *btot = the totals.
__device__ __forceinline__ void block_scan2(double& a, double& b, double (*wtot)[kWaves], double* atot, double* btot) {
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    for (int o = 1; o < 64; o <<= 1) {
        const double ua = __shfl_up(a, o), ub = __shfl_up(b, o);
        if (lane >= o) { a += ua; b += ub; }
    }
    if (lane == 63) { wtot[0][wv] = a; wtot[1][wv] = b; }
    __syncthreads();
    double pa = 0.0, pb = 0.0, ta = 0.0, tb = 0.0;
    for (int w = 0; w < kWaves; ++w) {
        if (w < wv) { pa += wtot[0][w]; pb += wtot[1][w]; }
        ta += wtot[0][w]; tb += wtot[1][w];
    }
    a += pa; b += pb; *atot = ta; *btot = tb;
    __syncthreads();
}

__global__ __launch_bounds__(kThreads) void sweep_kernel(SweepParams sw) {
    __shared__ SweepLds L;
    const int tid = threadIdx.x, row = blockIdx.x;
    const int cells = sw.nk * sw.nn;
    float* out = sw.accept_prob + static_cast<size_t>(row) * cells;

    // ---- merge the slices (same per-slice records as the solve kernel reads)
    int total = 0, bad = 0;
    double ptot = 0.0, qtot = 0.0;
    for (int s = 0; s < sw.splits; ++s) {
        total += sw.cand_count[row * sw.splits + s];
        bad |= sw.part_bad[row * sw.splits + s];
        ptot += sw.part_psum[row * sw.splits + s];
        qtot += sw.part_qsum[row * sw.splits + s];
    }
    if (bad || !(fabs(ptot - 1.0) <= 1e-3) || !(fabs(qtot - 1.0) <= 1e-3) || total <= 0 || total > kSelCap) {
        for (int c = tid; c < cells; c += kThreads) out[c] = __uint_as_float(0x7fc00000u);
        if (tid == 0) sw.status[row] = GR_ROW_BAD;
        return;
    }
    {
        int off = 0;
        for (int s = 0; s < sw.splits; ++s) {
            const int c = sw.cand_count[row * sw.splits + s];
            const unsigned long long* src = sw.cand + (static_cast<size_t>(row) * sw.splits + s) * kMaxSupport;
            for (int i = tid; i < c; i += kThreads) L.keys[off + i] = src[i];
            off += c;
        }
    }
    if (tid == 0) L.count = 0;
    __syncthreads();
    unsigned long long theta = 0ull;
    if (total > sw.kmax) theta = block_kth_largest<kThreads>(L.keys, total, sw.kmax, L.hist, L.pick);
    const int kk = min(total, sw.kmax);                       // <= kMaxSupport = kThreads
    for (int i = tid; i < total; i += kThreads) {
        const unsigned long long key = L.keys[i];
        if (key >= theta) {
            const int slot = atomicAdd(&L.count, 1);
            if (slot < kMaxSupport) L.ckey[slot] = key;
        }
    }
    __syncthreads();
    // ---- per slot: token id, q, p; rank by decreasing q (keys are distinct: ties go to the lower id)
    int qrank = 0, id = 0;
    if (tid < kk) {
        const unsigned long long mine = L.ckey[tid];
        id = key_id(mine);
        L.ids[tid] = id;
        L.qv[tid] = static_cast<double>(key_q(mine));
        L.pv[tid] = static_cast<double>(sw.p[static_cast<size_t>(row) * sw.V + id]);
        for (int j = 0; j < kk; ++j) qrank += static_cast<int>(L.ckey[j] > mine);
    }
    __syncthreads();
    // ---- rank by decreasing q/p: exact cross products (float x float fits a double), ties by id
    if (tid < kk) {
        const double qa = L.qv[tid], pa = L.pv[tid];
        int rank = 0;
        for (int j = 0; j < kk; ++j) {
            const double lhs = L.qv[j] * pa, rhs = qa * L.pv[j];              // j before me?
            rank += static_cast<int>(lhs > rhs) | (static_cast<int>(lhs == rhs) & static_cast<int>(L.ids[j] < id));
        }
        L.rp[rank] = pa / ptot; L.rq[rank] = qa; L.rqr[rank] = qrank;
    }
    __syncthreads();
    // ---- the grid: for each k the masked prefix sums along the order, for each n the best prefix
    const bool have = tid < kk;
    const double myp = have ? L.rp[tid] : 0.0, myq = have ? L.rq[tid] : 0.0;
    const int myqr = have ? L.rqr[tid] : 0x7fffffff;
    for (int a = 0; a < sw.nk; ++a) {
        const bool on = myqr < sw.ks[a];
        double P = on ? myp : 0.0, S = on ? myq : 0.0, Ptot, Stot;
        block_scan2(P, S, L.wtot, &Ptot, &Stot);
        const double Q = S / Stot;                            // Stot > 0: the largest q is positive
        // a rank outside this support repeats the prefix before it (or the empty prefix, F = 0);
        // the minima of all draft counts meet in LDS behind one barrier
        for (int b = 0; b < sw.nn; ++b) {
            const double F = have ? P - ipow(Q, sw.ns[b]) : 0.0;
            const double m = wave_min(fmin(F, 0.0));
            if ((tid & 63) == 0) L.cell[b][tid >> 6] = m;
        }
        __syncthreads();
        if (tid < sw.nn) {
            double t = L.cell[tid][0];
            for (int w = 1; w < kWaves; ++w) t = fmin(t, L.cell[tid][w]);
            out[a * sw.nn + tid] = static_cast<float>(1.0 + t);
        }
        // L.cell is written again only behind the two barriers of the next scan
    }
    if (tid == 0) sw.status[row] = GR_ROW_OK;
}

}  // namespace

hipError_t launch_sweep(const SweepParams& sw, int B, hipStream_t stream) {
    hipLaunchKernelGGL(sweep_kernel, dim3(B), dim3(kThreads), 0, stream, sw);
    return hipGetLastError();
}

}  // namespace gr
