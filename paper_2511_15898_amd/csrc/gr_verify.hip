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
#include "gr_verify_row.h"

namespace gr {

namespace {

constexpr int KS = kMaxSupport;
constexpr int kTile = kThreads * 4;

// Residual weights of one tile of tokens [base, base + kTile) into LDS `w` (zero beyond V).
__device__ void tile_weights(double* w, const Slice& S, const RowInfo& info, const int* order,
                             const double* rho, const double* rho_id, const float* prow, int base, int V) {
    const int tid = threadIdx.x;
    if (rho_id && S.mode == kInner) {                   // full-vocabulary policy: residuals by token id
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int t = base + tid * 4 + j;
            w[tid * 4 + j] = t < V ? S.scale * rho_id[t] : 0.0;
        }
        __syncthreads();
        return;
    }
    const double f = S.scale / info.p_total;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int t = base + tid * 4 + j;
        w[tid * 4 + j] = t < V ? f * p_entry(prow, t, info) : 0.0;
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
    const float* __restrict__ p, int V, int n, PolicyView pv, const RowInfo* __restrict__ infos,
    const int* __restrict__ drafts, const float* __restrict__ uniforms, int* __restrict__ token,
    unsigned char* __restrict__ accepted) {
    __shared__ VerifyLds vl;
    const int row = blockIdx.x;
    const RowInfo info = infos[row];
    RowPolicy rp;
    rp.o = pv.order + static_cast<size_t>(row) * pv.stride;
    rp.bl = pv.block + static_cast<size_t>(row) * pv.stride;
    rp.wt = pv.weight + static_cast<size_t>(row) * pv.stride;
    rp.rh = pv.rho + static_cast<size_t>(row) * pv.stride;
    rp.rk = pv.rank_of ? pv.rank_of + static_cast<size_t>(row) * pv.stride : nullptr;
    rp.rid = pv.rho_id ? pv.rho_id + static_cast<size_t>(row) * pv.stride : nullptr;
    rp.pieces = pv.piece_psum ? pv.piece_psum + static_cast<size_t>(row) * pv.piece_stride : nullptr;
    rp.prefs = pv.piece_pref ? pv.piece_pref + static_cast<size_t>(row) * pv.piece_stride : nullptr;
    verify_row(vl, p + static_cast<size_t>(row) * V, V, n, rp, info, drafts + static_cast<size_t>(row) * n, uniforms[row],
               token + row, accepted + row);
}

__global__ __launch_bounds__(kThreads) void slice_kernel(
    const float* __restrict__ p, int V, int n, PolicyView pv, const RowInfo* __restrict__ infos,
    const int* __restrict__ drafts, float* __restrict__ pi, float* __restrict__ accept_given) {
    __shared__ Slice S;
    __shared__ double w[kTile];
    const int tid = threadIdx.x, row = blockIdx.x;
    const RowInfo info = infos[row];
    const float* prow = p + static_cast<size_t>(row) * V;
    float* out = pi + static_cast<size_t>(row) * V;
    const int* o = pv.order + static_cast<size_t>(row) * pv.stride;
    const int* rk = pv.rank_of ? pv.rank_of + static_cast<size_t>(row) * pv.stride : nullptr;
    const double* rid = pv.rho_id ? pv.rho_id + static_cast<size_t>(row) * pv.stride : nullptr;
    if (info.status == GR_ROW_BAD) {
        for (int t = tid; t < V; t += kThreads) out[t] = 0.f;
        if (tid == 0) accept_given[row] = 0.f;
        return;
    }
    build_slice(S, info, o, pv.block + static_cast<size_t>(row) * pv.stride, pv.weight + static_cast<size_t>(row) * pv.stride,
                rk, drafts + static_cast<size_t>(row) * n, n, prow, V);
    const bool spread = (S.mode == kInner || S.mode == kFallback) && S.scale > 0.0;
    for (int base = 0; base < V; base += kTile) {
        if (spread) {
            tile_weights(w, S, info, o, pv.rho + static_cast<size_t>(row) * pv.stride, rid, prow, base, V);
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

void launch_verify(const float* p, int B, int V, int n, const PolicyView& pv, const RowInfo* info, const int* drafts,
                   const float* uniforms, int* token, unsigned char* accepted, hipStream_t stream) {
    hipLaunchKernelGGL(verify_kernel, dim3(B), dim3(kThreads), 0, stream, p, V, n, pv, info, drafts, uniforms,
                       token, accepted);
}

void launch_slice(const float* p, int B, int V, int n, const PolicyView& pv, const RowInfo* info, const int* drafts,
                  float* pi, float* accept_given, hipStream_t stream) {
    hipLaunchKernelGGL(slice_kernel, dim3(B), dim3(kThreads), 0, stream, p, V, n, pv, info, drafts, pi, accept_given);
}

}  // namespace gr
