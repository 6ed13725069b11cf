// Streaming support selection: the only HBM-bound step of the verifier.
//
// Top-k draft sampling restricts the whole problem to the k tokens of largest q (App. "Top-k
// Sampling for the Relaxed OTLP"), so one pass over the p and q rows suffices: it keeps the k
// largest q per row slice, and the float64 row sums of p and q that normalise them later.
#include "gr_internal.h"

namespace gr {

// grid = (splits, B); workgroup (s, b) streams tokens [s*slice_len, min(V, (s+1)*slice_len)) of row b;
// slice_len is a multiple of the tile (1024 tokens).
// Candidates are 64-bit keys (q bits, ~id) appended to an LDS buffer while they exceed the current
// threshold; when a further tile might overflow the buffer it is cut back to its k largest keys and
// the threshold is raised to the k-th.  The buffer never overflows: before each tile it holds at most
// kSelCap - kSelTile keys and a tile appends at most kSelTile.
__global__ __launch_bounds__(kThreads) void select_kernel(
    const float* __restrict__ p, const float* __restrict__ q, int V, int k, int slice_len,
    unsigned long long* __restrict__ cand, int* __restrict__ cand_count,
    double* __restrict__ part_psum, double* __restrict__ part_qsum, int* __restrict__ part_bad,
    double* __restrict__ piece_psum, int piece_stride) {
    __shared__ unsigned long long keys[kSelCap];
    __shared__ int hist[256];
    __shared__ int pick[4];
    __shared__ int count;
    __shared__ double red[kWaves];

    const int tid = threadIdx.x;
    const int s = blockIdx.x, b = blockIdx.y, splits = gridDim.x;
    const int v0 = s * slice_len;
    const int v1 = min(V, v0 + slice_len);
    const float* qr = q + static_cast<size_t>(b) * V;
    const float* pr = p + static_cast<size_t>(b) * V;
    // float4 loads need 16-byte aligned rows: V % 4 == 0 (slice_len is a multiple of 4).
    const bool vec = (V & 3) == 0 && ((reinterpret_cast<uintptr_t>(p) | reinterpret_cast<uintptr_t>(q)) & 15) == 0;

    if (tid == 0) count = 0;
    __syncthreads();

    // threshold: keys above it are candidates.  Start just below the smallest positive q.
    unsigned long long theta = 0x00000000FFFFFFFFull;
    double ps = 0.0, qs = 0.0;
    int bad = 0;

    for (int base = v0; base < v1; base += kSelTile) {
        const int i0 = base + tid * 4;
        float qv[4], pv[4];
        if (vec && i0 + 3 < v1) {
            const float4 q4 = *reinterpret_cast<const float4*>(qr + i0);
            const float4 p4 = *reinterpret_cast<const float4*>(pr + i0);
            qv[0] = q4.x; qv[1] = q4.y; qv[2] = q4.z; qv[3] = q4.w;
            pv[0] = p4.x; pv[1] = p4.y; pv[2] = p4.z; pv[3] = p4.w;
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const bool in = i0 + j < v1;
                qv[j] = in ? qr[i0 + j] : 0.f;
                pv[j] = in ? pr[i0 + j] : 0.f;
            }
        }
        // float64 sum of p over the 256 tokens this wave holds (slices start on tile boundaries, so the
        // pieces line up over the whole row): the rejection walk of the verify kernel starts from these
        {
            const double p4 = (static_cast<double>(pv[0]) + static_cast<double>(pv[1])) +
                              (static_cast<double>(pv[2]) + static_cast<double>(pv[3]));
            const double pw = wave_sum(p4);
            if (piece_psum && (tid & 63) == 0) piece_psum[static_cast<size_t>(b) * piece_stride + (base >> 8) + (tid >> 6)] = pw;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            bad |= !(qv[j] >= 0.f) | !(pv[j] >= 0.f);          // NaN or negative
            ps += static_cast<double>(pv[j]);
            qs += static_cast<double>(qv[j]);
            const unsigned long long key = make_key(qv[j], i0 + j);
            if (qv[j] > 0.f && key > theta) {
                const int slot = atomicAdd(&count, 1);
                keys[slot] = key;                                  // slot < kSelCap by construction
            }
        }
        __syncthreads();
        const int c = count;
        __syncthreads();
        if (c + kSelTile > kSelCap && c > k) {
            theta = block_kth_largest(keys, c, k, hist, pick);
            // keep the k keys >= theta, in place: read all, then write the survivors
            unsigned long long mine[kSelCap / kThreads];
#pragma unroll
            for (int r = 0; r < kSelCap / kThreads; ++r) {
                const int i = tid + r * kThreads;
                mine[r] = i < c ? keys[i] : 0ull;
            }
            __syncthreads();
            if (tid == 0) count = 0;
            __syncthreads();
#pragma unroll
            for (int r = 0; r < kSelCap / kThreads; ++r)
                if (mine[r] >= theta && mine[r] != 0ull) keys[atomicAdd(&count, 1)] = mine[r];
            __syncthreads();
        }
    }

    int c = count;
    __syncthreads();
    if (c > k) {
        theta = block_kth_largest(keys, c, k, hist, pick);
    } else {
        theta = 0ull;
    }
    // emit the keys >= theta (at most k of them)
    unsigned long long* out = cand + (static_cast<size_t>(b) * splits + s) * kMaxSupport;
    if (tid == 0) pick[0] = 0;
    __syncthreads();
    for (int i = tid; i < c; i += kThreads) {
        const unsigned long long key = keys[i];
        if (key >= theta) {
            const int slot = atomicAdd(&pick[0], 1);
            if (slot < kMaxSupport) out[slot] = key;
        }
    }
    __syncthreads();
    const double pt = block_sum(ps, red);
    const double qt = block_sum(qs, red);
    const int anybad = block_sum_i(bad, red);
    if (tid == 0) {
        cand_count[b * splits + s] = min(pick[0], kMaxSupport);
        part_psum[b * splits + s] = pt;
        part_qsum[b * splits + s] = qt;
        part_bad[b * splits + s] = anybad;
    }
}

void launch_select(const float* p, const float* q, int B, int V, int k, int splits, int slice_len,
                   unsigned long long* cand, int* cand_count, double* psum, double* qsum, int* bad,
                   double* piece_psum, int piece_stride, hipStream_t stream) {
    dim3 grid(splits, B);
    hipLaunchKernelGGL(select_kernel, grid, dim3(kThreads), 0, stream, p, q, V, k, slice_len, cand,
                       cand_count, psum, qsum, bad, piece_psum, piece_stride);
}

}  // namespace gr
