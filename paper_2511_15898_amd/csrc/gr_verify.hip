// Transport slice pi(.|drafts) and the single inverse-CDF draw from it.
//
// Given the drafted tuple omega (Eq. "cases", Eq. "approx-c", normalised by pdraft(omega)):
//   omega in (H*)^n : pi(i) = w_i / (1 + sum_{j in set(omega)} w_j) for the drafted tokens, and the
//                     slack 1/(1 + sum) is spread over the tokens outside H* in proportion to their
//                     residuals p(i) - p_i (the residual lift of Eq. (3));
//   otherwise       : all mass stays on the drafted tokens of the block that holds the lowest-ratio
//                     draft, softmax of that block's weights.
// Rows whose solve failed use pi = p.  One 256-thread workgroup per row.
#include "gr_internal.h"

namespace gr {

namespace {

constexpr int KS = kMaxSupport;
constexpr int kTile = kThreads * 4;

enum Mode { kOuter = 0, kInner = 1, kFallback = 2, kBadDraft = 3 };

struct Slice {
    int nd;                    // number of distinct drafts
    int tok[GR_MAX_N];         // in order of first appearance
    int pos[GR_MAX_N];         // rank position in the support, -1 if absent
    double pi[GR_MAX_N];       // probability of each distinct draft
    double acc;                // sum of pi over the drafts
    double scale;              // multiplies the residual weight of every other token
    int mode;
};

// All threads call; result in LDS `S`.  order/block/weight: this row's policy arrays.
__device__ void build_slice(Slice& S, const RowInfo& info, const int* order, const int* block,
                            const double* weight, const int* drafts, int n, const float* prow, int V) {
    const int tid = threadIdx.x;
    if (tid == 0) {
        int nd = 0;
        S.mode = kOuter;
        for (int i = 0; i < n; ++i) {
            const int t = drafts[i];
            if (t < 0 || t >= V) { S.mode = kBadDraft; continue; }
            bool seen = false;
            for (int j = 0; j < nd; ++j) seen |= (S.tok[j] == t);
            if (!seen) { S.tok[nd] = t; S.pos[nd] = -1; ++nd; }
        }
        S.nd = nd;
    }
    __syncthreads();
    const int kk = info.support;
    if (info.status == GR_ROW_OK && tid < kk) {
        const int t = order[tid];
        for (int i = 0; i < S.nd; ++i) if (S.tok[i] == t) S.pos[i] = tid;
    }
    __syncthreads();
    if (tid == 0) {
        const int nd = S.nd;
        if (S.mode == kBadDraft) {
            for (int i = 0; i < nd; ++i) S.pi[i] = 0.0;
            S.acc = 0.0; S.scale = 0.0;
        } else if (info.status != GR_ROW_OK) {
            double a = 0.0;
            for (int i = 0; i < nd; ++i) { S.pi[i] = static_cast<double>(prow[S.tok[i]]) / info.p_total; a += S.pi[i]; }
            S.acc = a; S.scale = 1.0; S.mode = kFallback;
        } else {
            int mmax = -1; bool missing = false;
            for (int i = 0; i < nd; ++i) { missing |= S.pos[i] < 0; mmax = max(mmax, S.pos[i]); }
            if (missing) {
                for (int i = 0; i < nd; ++i) S.pi[i] = 0.0;
                S.acc = 0.0; S.scale = 0.0; S.mode = kBadDraft;
            } else if (mmax < info.h) {
                double s = 0.0;
                for (int i = 0; i < nd; ++i) s += weight[S.pos[i]];
                const double den = 1.0 + s;
                for (int i = 0; i < nd; ++i) S.pi[i] = weight[S.pos[i]] / den;
                S.acc = 1.0 - 1.0 / den;
                S.scale = info.res_total > 0.0 ? (1.0 / den) / info.res_total : 0.0;
                S.mode = kInner;
            } else {
                const int b = block[mmax];
                double s = 0.0; int members = 0;
                for (int i = 0; i < nd; ++i)
                    if (S.pos[i] >= info.h && block[S.pos[i]] == b) { s += weight[S.pos[i]]; ++members; }
                for (int i = 0; i < nd; ++i) {
                    const bool in = S.pos[i] >= info.h && block[S.pos[i]] == b;
                    S.pi[i] = in ? (s > 0.0 ? weight[S.pos[i]] / s : 1.0 / members) : 0.0;
                }
                S.acc = 1.0; S.scale = 0.0; S.mode = kOuter;
            }
        }
    }
    __syncthreads();
}

// Residual weights of one tile of tokens [base, base + kTile) into LDS `w` (zero beyond V).
__device__ void tile_weights(double* w, const Slice& S, const RowInfo& info, const int* order,
                             const double* rho, const float* prow, int base, int V) {
    const int tid = threadIdx.x;
    const double f = S.scale / info.p_total;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int t = base + tid * 4 + j;
        w[tid * 4 + j] = t < V ? f * static_cast<double>(prow[t]) : 0.0;
    }
    __syncthreads();
    if (S.mode == kInner) {
        if (tid < info.support) {                       // support tokens: residual rho outside H*, none inside
            const int t = order[tid] - base;
            if (t >= 0 && t < kTile) w[t] = tid >= info.h ? S.scale * rho[tid] : 0.0;
        }
    } else if (tid < S.nd) {                            // fallback: the drafts were listed first
        const int t = S.tok[tid] - base;
        if (t >= 0 && t < kTile) w[t] = 0.0;
    }
    __syncthreads();
}

}  // namespace

__global__ __launch_bounds__(kThreads) void verify_kernel(
    const float* __restrict__ p, int V, int n, const int* __restrict__ order, const int* __restrict__ block,
    const double* __restrict__ weight, const double* __restrict__ rho, const RowInfo* __restrict__ infos,
    const int* __restrict__ drafts, const float* __restrict__ uniforms, int* __restrict__ token,
    unsigned char* __restrict__ accepted) {
    __shared__ Slice S;
    __shared__ double w[kTile];
    __shared__ double red[kWaves];
    __shared__ double wtot[kWaves];
    __shared__ int chosen;
    const int tid = threadIdx.x, row = blockIdx.x;
    const RowInfo info = infos[row];
    const float* prow = p + static_cast<size_t>(row) * V;
    const int* o = order + static_cast<size_t>(row) * KS;
    const int* bl = block + static_cast<size_t>(row) * KS;
    const double* wt = weight + static_cast<size_t>(row) * KS;
    const double* rh = rho + static_cast<size_t>(row) * KS;
    if (info.status == GR_ROW_BAD) {
        if (tid == 0) { token[row] = -1; accepted[row] = 0; }
        return;
    }
    build_slice(S, info, o, bl, wt, drafts + static_cast<size_t>(row) * n, n, prow, V);
    const double u = static_cast<double>(uniforms[row]);
    double c = 0.0;
    if (tid == 0) {
        int pickd = -1, last = -1;
        for (int i = 0; i < S.nd; ++i) {
            if (!(S.pi[i] > 0.0)) continue;
            c += S.pi[i]; last = S.tok[i];
            if (pickd < 0 && u < c) pickd = S.tok[i];
        }
        if (pickd < 0 && (S.mode == kOuter || S.scale == 0.0)) pickd = last;   // nothing beyond the drafts
        chosen = pickd;
        red[0] = c;
    }
    __syncthreads();
    c = red[0];
    const int first = chosen;
    __syncthreads();
    if (S.mode == kBadDraft) {
        if (tid == 0) { token[row] = -1; accepted[row] = 0; }
        return;
    }
    if (first >= 0) {
        if (tid == 0) { token[row] = first; accepted[row] = 1; }
        return;
    }
    // ---- not among the drafts: walk the remaining tokens by ascending id
    int last_pos = -1;                       // largest token id seen with positive weight
    int found = -1;
    for (int base = 0; base < V && found < 0; base += kTile) {
        tile_weights(w, S, info, o, rh, prow, base, V);
        double mine[4]; double s4 = 0.0;
#pragma unroll
        for (int j = 0; j < 4; ++j) { mine[j] = w[tid * 4 + j]; s4 += mine[j]; }
        // exclusive prefix of the per-thread sums
        double incl = s4;
        for (int off = 1; off < 64; off <<= 1) { const double up = __shfl_up(incl, off); if ((tid & 63) >= off) incl += up; }
        if ((tid & 63) == 63) wtot[tid >> 6] = incl;
        __syncthreads();
        double before = 0.0, tile_total = 0.0;
        for (int wv = 0; wv < kWaves; ++wv) { if (wv < (tid >> 6)) before += wtot[wv]; tile_total += wtot[wv]; }
        double run = c + before + (incl - s4);
        int hit = 0x7fffffff, lastp = -1;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (mine[j] > 0.0) {
                run += mine[j]; lastp = base + tid * 4 + j;
                if (hit == 0x7fffffff && u < run) hit = base + tid * 4 + j;
            }
        }
        const double hmin = block_min(static_cast<double>(hit), red);
        const double lmax = block_max(static_cast<double>(lastp), red);
        if (lmax >= 0.0) last_pos = static_cast<int>(lmax);
        if (hmin < 2147483647.0) found = static_cast<int>(hmin);
        c += tile_total;
        __syncthreads();
    }
    if (tid == 0) {
        int t = found >= 0 ? found : last_pos;
        bool acc = false;
        if (t < 0) {                          // no residual mass at all: keep the last draft with mass
            for (int i = 0; i < S.nd; ++i) if (S.pi[i] > 0.0) t = S.tok[i];
            acc = t >= 0;
        }
        token[row] = t; accepted[row] = acc ? 1 : 0;
    }
}

__global__ __launch_bounds__(kThreads) void slice_kernel(
    const float* __restrict__ p, int V, int n, const int* __restrict__ order, const int* __restrict__ block,
    const double* __restrict__ weight, const double* __restrict__ rho, const RowInfo* __restrict__ infos,
    const int* __restrict__ drafts, float* __restrict__ pi, float* __restrict__ accept_given) {
    __shared__ Slice S;
    __shared__ double w[kTile];
    const int tid = threadIdx.x, row = blockIdx.x;
    const RowInfo info = infos[row];
    const float* prow = p + static_cast<size_t>(row) * V;
    float* out = pi + static_cast<size_t>(row) * V;
    const int* o = order + static_cast<size_t>(row) * KS;
    if (info.status == GR_ROW_BAD) {
        for (int t = tid; t < V; t += kThreads) out[t] = 0.f;
        if (tid == 0) accept_given[row] = 0.f;
        return;
    }
    build_slice(S, info, o, block + static_cast<size_t>(row) * KS, weight + static_cast<size_t>(row) * KS,
                drafts + static_cast<size_t>(row) * n, n, prow, V);
    const bool spread = (S.mode == kInner || S.mode == kFallback) && S.scale > 0.0;
    for (int base = 0; base < V; base += kTile) {
        if (spread) {
            tile_weights(w, S, info, o, rho + static_cast<size_t>(row) * KS, prow, base, V);
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) w[tid * 4 + j] = 0.0;
            __syncthreads();
        }
        if (tid < S.nd) {                    // the drafts themselves
            const int t = S.tok[tid] - base;
            if (t >= 0 && t < kTile) w[t] = S.pi[tid];
        }
        __syncthreads();
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int t = base + tid * 4 + j;
            if (t < V) out[t] = static_cast<float>(w[tid * 4 + j]);
        }
        __syncthreads();
    }
    if (tid == 0) accept_given[row] = static_cast<float>(S.acc);
}

void launch_verify(const float* p, int B, int V, int n, const int* order, const int* block,
                   const double* weight, const double* rho, const RowInfo* info, const int* drafts,
                   const float* uniforms, int* token, unsigned char* accepted, hipStream_t stream) {
    hipLaunchKernelGGL(verify_kernel, dim3(B), dim3(kThreads), 0, stream, p, V, n, order, block, weight,
                       rho, info, drafts, uniforms, token, accepted);
}

void launch_slice(const float* p, int B, int V, int n, const int* order, const int* block,
                  const double* weight, const double* rho, const RowInfo* info, const int* drafts,
                  float* pi, float* accept_given, hipStream_t stream) {
    hipLaunchKernelGGL(slice_kernel, dim3(B), dim3(kThreads), 0, stream, p, V, n, order, block, weight,
                       rho, info, drafts, pi, accept_given);
}

}  // namespace gr
