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
//
// LOGITS: p and q are the target and draft logits and `temperature` [B] the sampling temperature of each row
// (App. A: temperature only changes how p and q come from the logits).  The k largest q are the k largest
// draft logits, so the keys carry the draft logit (as a monotone 32-bit pattern); the draft needs no
// normaliser, because q is renormalised over the support anyway.  The target's normaliser is an online
// softmax: every wave keeps a reference r (the largest target logit it has seen, raised tile by tile) and
// its lanes the float64 sums of exp((t - r) / T); part_psum / part_pref get the
// slice's sum and reference, piece_psum / piece_pref those of every 256 tokens.
template <bool LOGITS>
__global__ __launch_bounds__(kThreads, 8) void select_kernel(
    const float* __restrict__ p, const float* __restrict__ q, int V, int k, int slice_len,
    unsigned long long* __restrict__ cand, int* __restrict__ cand_count,
    double* __restrict__ part_psum, double* __restrict__ part_qsum, int* __restrict__ part_bad,
    double* __restrict__ piece_psum, int piece_stride,
    const float* __restrict__ temperature, float* __restrict__ part_pref, float* __restrict__ piece_pref) {
    __shared__ unsigned long long keys[kSelCap];
    __shared__ int hist[256];
    __shared__ int pick[4];
    __shared__ int count;
    __shared__ double red[kWaves];
    __shared__ float wref[kWaves];
    __shared__ double e2tab[32];                           // 2^(-j/32), the table of exp_neg (LOGITS only)

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
    // LOGITS: a temperature that is not a positive finite number marks the row bad
    double inv_temp = 0.0;
    float scale2 = 0.f;                                    // log2(e) / T
    float theta_d = -__builtin_inff();                    // the draft logit of the threshold key
    float ref = -__builtin_inff();
    if (LOGITS) {
        const float T = temperature[b];
        if (!(T > 0.f) || !(T <= 3.0e38f)) bad = 1; else { inv_temp = 1.0 / static_cast<double>(T); scale2 = 1.44269504088896341f / T; }
        if (tid < 32) e2tab[tid] = exp2(-static_cast<double>(tid) / 32.0);
        __syncthreads();
    }

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
        if (LOGITS) {
            // Entries beyond the slice read as -inf (no mass, never a candidate), like a masked token.  A NaN or a
            // +inf anywhere makes the sum of the eight values NaN or +inf and marks the row bad (so do finite
            // logits beyond 3e37, which no model emits).  Then the wave's reference rises to the largest target
            // logit of the tile, the sums so far are rescaled, and the tile's terms are added.
            if (!(vec && i0 + 3 < v1)) {
#pragma unroll
                for (int j = 0; j < 4; ++j) if (!(i0 + j < v1)) { pv[j] = -__builtin_inff(); qv[j] = -__builtin_inff(); }
            }
            const float probe = ((pv[0] + pv[1]) + (pv[2] + pv[3])) + ((qv[0] + qv[1]) + (qv[2] + qv[3]));
            bad |= !(probe < 3.0e38f);
            float m4 = fmaxf(fmaxf(pv[0], pv[1]), fmaxf(pv[2], pv[3]));
            if (__any(m4 > ref)) {                                 // the wave's reference rises (rare after the first tiles)
#pragma unroll
                for (int o = 1; o < 64; o <<= 1) m4 = fmaxf(m4, __shfl_xor(m4, o));
                ps = (ref > -3.0e38f) ? ps * exp_neg((static_cast<double>(m4) - static_cast<double>(ref)) * inv_temp, e2tab) : 0.0;
                ref = m4;
            }
            // Terms more than 25 temperatures below the reference (each below 1.4e-11 of it) take the hardware's
            // float32 exponential: their relative error of 1e-7 moves the sum by at most 1.4e-18 V of the reference's
            // own term (2e-13 at V = 128256).  The others go through the float64 routine, one per lane and round
            // (few lanes hold any).
            double e4 = 0.0;
            if (ref > -3.0e38f) {
                const double r = static_cast<double>(ref);
                unsigned pend = 0u;
                float fs = 0.f;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float a = (pv[j] - ref) * scale2;                // log2 of the term; -inf for a masked entry
                    const bool near = a >= -36.0673760222f;                // 25 temperatures, in bits
                    const float f = __builtin_amdgcn_exp2f(a);                 // the bare instruction: results below 2^-126 flush to 0, which is what they are worth here
                    fs += near ? 0.f : f;                                  // each below 1.4e-11: float32 adds lose nothing that matters
                    pend |= near ? (1u << j) : 0u;
                }
                e4 = static_cast<double>(fs);
                while (__any(pend != 0u)) {
                    if (pend != 0u) {
                        const int j = __ffs(static_cast<int>(pend)) - 1;
                        const float tj = j == 0 ? pv[0] : (j == 1 ? pv[1] : (j == 2 ? pv[2] : pv[3]));
                        e4 += exp_neg((r - static_cast<double>(tj)) * inv_temp, e2tab);
                        pend &= pend - 1u;
                    }
                }
            }
            ps += e4;
            // the pieces' sums only steer the rejection walk (1e-7 relative is plenty): float32 reduction
            const float pw = wave_sum_f32(static_cast<float>(e4));
            if (piece_psum && (tid & 63) == 0) {
                const size_t at = static_cast<size_t>(b) * piece_stride + (base >> 8) + (tid >> 6);
                piece_psum[at] = static_cast<double>(pw); piece_pref[at] = ref;
            }
            // candidates: the draft logit against the threshold's own logit first, the full key (ties by id) only then
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (qv[j] >= theta_d && qv[j] > -3.0e38f) {
                    const unsigned long long key = make_key_logit(qv[j], i0 + j);
                    if (key > theta) {
                        const int slot = atomicAdd(&count, 1);
                        keys[slot] = key;                          // slot < kSelCap by construction
                    }
                }
            }
        } else {
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
        }
        __syncthreads();
        const int c = count;
        __syncthreads();
        if (c + kSelTile > kSelCap && c > k) {
            theta = block_kth_largest(keys, c, k, hist, pick);
            if (LOGITS) theta_d = key_logit(theta);
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
    double pt, qt;
    float slice_ref = 0.f;
    if (LOGITS) {
        // the waves' sums, each relative to its own reference, brought to the slice's largest reference
        if ((tid & 63) == 0) wref[tid >> 6] = ref;
        __syncthreads();
        slice_ref = fmaxf(fmaxf(wref[0], wref[1]), fmaxf(wref[2], wref[3]));
        const double mine = (ref > -3.0e38f) ? ps * exp_neg((static_cast<double>(slice_ref) - static_cast<double>(ref)) * inv_temp, e2tab) : 0.0;
        pt = block_sum(mine, red);
        qt = 1.0;
    } else {
        pt = block_sum(ps, red);
        qt = block_sum(qs, red);
    }
    const int anybad = block_sum_i(bad, red);
    if (tid == 0) {
        cand_count[b * splits + s] = min(pick[0], kMaxSupport);
        part_psum[b * splits + s] = pt;
        part_qsum[b * splits + s] = qt;
        part_bad[b * splits + s] = anybad;
        if (LOGITS) part_pref[b * splits + s] = slice_ref;
    }
}

void launch_select(const float* p, const float* q, int B, int V, int k, int splits, int slice_len,
                   unsigned long long* cand, int* cand_count, double* psum, double* qsum, int* bad,
                   double* piece_psum, int piece_stride, hipStream_t stream) {
    dim3 grid(splits, B);
    hipLaunchKernelGGL(select_kernel<false>, grid, dim3(kThreads), 0, stream, p, q, V, k, slice_len, cand,
                       cand_count, psum, qsum, bad, piece_psum, piece_stride, nullptr, nullptr, nullptr);
}

void launch_select_logits(const float* target_logits, const float* draft_logits, const float* temperature, int B, int V, int k,
                          int splits, int slice_len, unsigned long long* cand, int* cand_count, double* psum, double* qsum,
                          int* bad, float* part_pref, double* piece_psum, float* piece_pref, int piece_stride, hipStream_t stream) {
    dim3 grid(splits, B);
    hipLaunchKernelGGL(select_kernel<true>, grid, dim3(kThreads), 0, stream, target_logits, draft_logits, V, k, slice_len, cand,
                       cand_count, psum, qsum, bad, piece_psum, piece_stride, temperature, part_pref, piece_pref);
}

}  // namespace gr
