// Internal declarations shared by the kernels and the C ABI of the Global Resolution verifier.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gr_verify.h"

namespace gr {

constexpr int kThreads = 256;             // every kernel here runs 256-thread workgroups (4 wave64)
constexpr int kWaves = kThreads / 64;
constexpr int kMaxSupport = GR_MAX_SUPPORT;
constexpr int kMaxT = GR_MAX_T;
constexpr int kSelTile = kThreads * 4;    // tokens per streaming tile (one float4 per thread)
constexpr int kSelCap = 2048;             // candidate keys held in LDS (>= kMaxSupport + kSelTile)
constexpr int kMaxSplits = 8;             // workgroups that share one row in the select kernel
constexpr int kHist = 5;                  // Anderson history length (current + 4)

// Per-row result of the solve kernel (one per row, in HBM).
struct RowInfo {
    int support;        // k' = |V_0|
    int h;              // |H*|
    int status;         // GR_ROW_*
    int iterations;     // fixed-point evaluations summed over the row's programs
    double alpha_star;  // 1 + psi(H*)
    double res_total;   // sum of residuals p(i) - p_i over tokens outside H* (= 1 - alpha*)
    double p_total;     // float64 row sum of p
    double q_total;     // float64 row sum of q (before top-k)
    double node_tokens; // sum over evaluator calls of (quadrature nodes x active tokens)
    double p_ref;       // rows given as logits: p(i) = exp((t_i - p_ref) inv_temp) / p_total ...
    double inv_temp;    // ... with inv_temp = 1 / temperature; 0 for rows given as probabilities
    double q_ref;       // rows given as logits on the HBM-resident path: q(i) proportional to exp((d_i - q_ref) inv_temp)
#ifdef GR_PHASE_CLOCKS
    long long clk[24];  // shader-clock cycles of thread 0 per phase of the solve kernel (profiling builds only)
    double errlog[24];  // stopping measure after each of the first evaluations
#endif
};

struct SolveParams {
    const float* p; const float* q;
    int B, V, n, k, splits;
    double tau;         // the paper's error threshold, float32 value widened
    double rel_tol;
    double tail_mass;   // nucleus cut of the draft (0: none)
    int max_iter, max_T;
    // select kernel output
    const unsigned long long* cand;   // [B, splits, kMaxSupport] keys
    const int* cand_count;            // [B, splits]
    const double* part_psum;          // [B, splits]
    const double* part_qsum;          // [B, splits]
    const int* part_bad;              // [B, splits]
    // rows given as logits (p = target logits, q unused): temperature [B], the slices' softmax references [B, splits]
    int logits; const float* temperature; const float* part_pref;
    const float* draft_temperature;   // [B] the draft's own temperature, or nullptr: the row's temperature serves both models
    // policy object
    int* order; int* block; double* weight; double* rho; double* pnorm;   // [B, kMaxSupport]
    RowInfo* info;                    // [B]
    float* accept_prob; int* status;  // caller's outputs [B]
    double* newton_ws;                // [B, kMaxT * (kMaxT + 1)] Jacobian scratch of the Newton fallback
    // verification in the same launch (v_drafts == nullptr: none): drafts [B, n], uniforms [B] -> token [B], accepted [B];
    // the sums of p over pieces of 256 tokens that the select pass left, as in PolicyView
    const int* v_drafts; const float* v_uniforms; int* v_token; unsigned char* v_accepted;
    const double* piece_psum; int piece_stride; const float* piece_pref;
};

// Workspace and arguments of the full-vocabulary path (no top-k).  Per-token arrays are row-major with
// stride V + 2; P, Q, F, G hold kk + 1 entries per row (prefix index 0..kk), blo the record positions.
struct FullParams {
    const float* p; const float* q;
    int B, V, n, max_T, max_iter;
    int k;             // top-k on q (V: none)
    double tau, rel_tol;
    double tail_mass;  // nucleus cut of the draft: share of the draw mass that may be left out (0: none)
    int logits; const float* temperature;   // rows given as logits (p = target logits, q = draft logits), one temperature per row
    const float* draft_temperature;         // [B] the draft's own temperature, or nullptr
    unsigned long long* key0; unsigned long long* key1; int* val0; int* val1;   // sort buffers
    int* order;        // token ids by decreasing q/p
    int* byq;          // ranks by (inside H* first, decreasing q, token id)
    double* pn; double* qn; double* P; double* Q; double* F; double* rho; double* tgt; double* weight;
    int* flag; int* blk; int* blo; int* inT; int* bcount;
    int* rank_of;      // [B, V + 2] rank of each token id, -1 outside the support
    double* rho_id;    // [B, V + 2] residual p(i) - p_i by token id (0 inside H*)
    int* nblk;         // [B] number of outer blocks
    int* tcount;       // [B, 2] sizes of the two truncation sets
    RowInfo* info; float* accept_prob; int* status;
    double* newton_ws; // [B, kMaxT * (kMaxT + 1)] Jacobian scratch of the Newton fallback
};
constexpr size_t kFullBytesPerToken = 2 * 8 + 2 * 4 + 2 * 4 + 8 * 8 + 5 * 4 + 4 + 8;

void launch_full_prologue(const FullParams& fp, hipStream_t stream);
struct FullSweep;
void launch_full_sweep(const FullParams& fp, const FullSweep& fs, hipStream_t stream);
void launch_select(const float* p, const float* q, int B, int V, int k, int splits, int slice_len,
                   unsigned long long* cand, int* cand_count, double* psum, double* qsum, int* bad,
                   double* piece_psum, int piece_stride, hipStream_t stream);
void launch_select_logits(const float* target_logits, const float* draft_logits, const float* temperature, int B, int V, int k,
                          int splits, int slice_len, unsigned long long* cand, int* cand_count, double* psum, double* qsum,
                          int* bad, float* part_pref, double* piece_psum, float* piece_pref, int piece_stride, hipStream_t stream);
hipError_t launch_solve(const SolveParams& sp, hipStream_t stream);
// The policy object as the verify and slice kernels read it.  Top-k policies: arrays [B, stride] with
// stride = kMaxSupport, rank_of = rho_id = nullptr.  Full-vocabulary policies: stride = V + 2, plus the
// rank of every token id and the residuals by token id.
struct PolicyView {
    const int* order; const int* block; const double* weight; const double* rho;
    const int* rank_of; const double* rho_id;
    size_t stride;
    const double* piece_psum;   // [B, piece_stride] float64 sums of p over pieces of 256 tokens, or nullptr
    int piece_stride;
    const float* piece_pref;    // rows given as logits: the reference each piece sum is relative to
};
void launch_verify(const float* p, int B, int V, int n, const PolicyView& pv, const RowInfo* info, const int* drafts,
                   const float* uniforms, int* token, unsigned char* accepted, hipStream_t stream);
void launch_slice(const float* p, int B, int V, int n, const PolicyView& pv, const RowInfo* info, const int* drafts,
                  float* pi, float* accept_given, hipStream_t stream);
hipError_t launch_full_programs(const FullParams& fp, hipStream_t stream);

// Acceptance-only sweep over a grid of top-k sizes and draft counts (one selection pass with kmax).
constexpr int kSweepMaxK = 8;     // top-k sizes per call
constexpr int kSweepMaxN = 16;    // draft counts per call
constexpr int kSweepMaxDrafts = 64;
struct SweepParams {
    const float* p; int V; int splits;
    const unsigned long long* cand; const int* cand_count;
    const double* part_psum; const double* part_qsum; const int* part_bad;
    int kmax, nk, nn;
    int ks[kSweepMaxK]; int ns[kSweepMaxN];
    float* accept_prob;           // [B, nk, nn]
    int* status;                  // [B]
};
hipError_t launch_sweep(const SweepParams& sw, int B, hipStream_t stream);
// The grid of a sweep whose largest support lives in the HBM workspace.
struct FullSweep {
    int nk, nn;
    int ks[kSweepMaxK]; int ns[kSweepMaxN];   // ks: V for "no top-k"
    double* mass;                 // [B, kSweepMaxK] q mass of each top-k support
    float* accept_prob;           // [B, nk, nn]
    int* status;                  // [B]
};
hipError_t solve_kernel_setup();

// ---------------------------------------------------------------- device helpers
// Wave reductions on the data-parallel-primitive path (no LDS round trip): a butterfly inside each
// row of 16 lanes (quad permutes, half-row mirror, row mirror: every lane ends with its row's
// result), then the four row results are read as scalars and combined.  All 64 lanes must be active;
// the result is the same bit pattern in every lane.
template <int CTRL>
__device__ __forceinline__ double dpp_move(double v) {
    int lo = __double2loint(v), hi = __double2hiint(v);
    // every control used here reads a live lane in every lane, so the destination needs no initial value
    lo = __builtin_amdgcn_mov_dpp(lo, CTRL, 0xF, 0xF, true);
    hi = __builtin_amdgcn_mov_dpp(hi, CTRL, 0xF, 0xF, true);
    return __hiloint2double(hi, lo);
}
template <int CTRL>
__device__ __forceinline__ int dpp_move(int v) {
    return __builtin_amdgcn_mov_dpp(v, CTRL, 0xF, 0xF, true);
}
__device__ __forceinline__ double read_lane(double v, int lane) {
    const int lo = __builtin_amdgcn_readlane(__double2loint(v), lane);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(v), lane);
    return __hiloint2double(hi, lo);
}
constexpr int kDppXor1 = 0xB1, kDppXor2 = 0x4E, kDppHalfMirror = 0x141, kDppMirror = 0x140;

__device__ __forceinline__ double wave_sum(double v) {
    v += dpp_move<kDppXor1>(v);
    v += dpp_move<kDppXor2>(v);
    v += dpp_move<kDppHalfMirror>(v);
    v += dpp_move<kDppMirror>(v);
    return (read_lane(v, 0) + read_lane(v, 16)) + (read_lane(v, 32) + read_lane(v, 48));
}
// The float32 sum over the wave, for sums that need no more (one move and one add per level).
__device__ __forceinline__ float wave_sum_f32(float v) {
    v += __int_as_float(dpp_move<kDppXor1>(__float_as_int(v)));
    v += __int_as_float(dpp_move<kDppXor2>(__float_as_int(v)));
    v += __int_as_float(dpp_move<kDppHalfMirror>(__float_as_int(v)));
    v += __int_as_float(dpp_move<kDppMirror>(__float_as_int(v)));
    const int b = __float_as_int(v);
    return (__int_as_float(__builtin_amdgcn_readlane(b, 0)) + __int_as_float(__builtin_amdgcn_readlane(b, 16))) +
           (__int_as_float(__builtin_amdgcn_readlane(b, 32)) + __int_as_float(__builtin_amdgcn_readlane(b, 48)));
}
__device__ __forceinline__ double wave_max(double v) {
    v = fmax(v, dpp_move<kDppXor1>(v));
    v = fmax(v, dpp_move<kDppXor2>(v));
    v = fmax(v, dpp_move<kDppHalfMirror>(v));
    v = fmax(v, dpp_move<kDppMirror>(v));
    return fmax(fmax(read_lane(v, 0), read_lane(v, 16)), fmax(read_lane(v, 32), read_lane(v, 48)));
}
__device__ __forceinline__ double wave_min(double v) {
    v = fmin(v, dpp_move<kDppXor1>(v));
    v = fmin(v, dpp_move<kDppXor2>(v));
    v = fmin(v, dpp_move<kDppHalfMirror>(v));
    v = fmin(v, dpp_move<kDppMirror>(v));
    return fmin(fmin(read_lane(v, 0), read_lane(v, 16)), fmin(read_lane(v, 32), read_lane(v, 48)));
}
__device__ __forceinline__ int wave_sum_i(int v) {
    v += dpp_move<kDppXor1>(v);
    v += dpp_move<kDppXor2>(v);
    v += dpp_move<kDppHalfMirror>(v);
    v += dpp_move<kDppMirror>(v);
    return (__builtin_amdgcn_readlane(v, 0) + __builtin_amdgcn_readlane(v, 16)) +
           (__builtin_amdgcn_readlane(v, 32) + __builtin_amdgcn_readlane(v, 48));
}

// Workgroup reductions over NW waves.  `red` is an LDS array of at least NW doubles; both barriers are inside, so `red` may be reused right after the call.
template <int NW = kWaves>
__device__ __forceinline__ double block_sum(double v, double* red) {
    v = wave_sum(v);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    double t = red[0];
    for (int w = 1; w < NW; ++w) t += red[w];
    __syncthreads();
    return t;
}
template <int NW = kWaves>
__device__ __forceinline__ double block_max(double v, double* red) {
    v = wave_max(v);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    double t = red[0];
    for (int w = 1; w < NW; ++w) t = fmax(t, red[w]);
    __syncthreads();
    return t;
}
template <int NW = kWaves>
__device__ __forceinline__ double block_min(double v, double* red) {
    v = wave_min(v);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    double t = red[0];
    for (int w = 1; w < NW; ++w) t = fmin(t, red[w]);
    __syncthreads();
    return t;
}
template <int NW = kWaves>
__device__ __forceinline__ int block_sum_i(int v, double* red) {
    int* r = reinterpret_cast<int*>(red);
    v = wave_sum_i(v);
    if ((threadIdx.x & 63) == 0) r[threadIdx.x >> 6] = v;
    __syncthreads();
    int t = r[0];
    for (int w = 1; w < NW; ++w) t += r[w];
    __syncthreads();
    return t;
}

// Arithmetic whose rounding must not depend on the compiler: no contraction into fused multiply-adds.
#pragma clang fp contract(off)
__device__ __forceinline__ double ipow(double x, int n) {
    double r = x;
    for (int i = 1; i < n; ++i) r = r * x;
    return r;
}

// a^n - (a-d)^n without cancellation: d * sum_{i<n} a^(n-1-i) b^i with b = a - d, by the
// recurrence s_i = a s_{i-1} + b^i (all terms nonnegative).
__device__ __forceinline__ double pow_diff(double a, double d, int n) {
    const double b = a - d;
    double s = 1.0, bp = 1.0;
    for (int i = 1; i < n; ++i) { bp = bp * b; s = s * a + bp; }
    return d * s;
}

// Inclusive prefix sums of x[0..count) in index order, added one after the other exactly as a
// sequential loop would (so the rounding does not depend on the machine), but held in the
// registers of one wave: lane j of round r owns element 64 r + j, the running sum travels through
// v_readlane.  Called by one whole wave; out[0] = start, out[i + 1] = start + x[0] + ... + x[i].
__device__ __forceinline__ void wave_sequential_scan(const double* x, double* out, int count, double start) {
    const int lane = threadIdx.x & 63;
    double acc = start;
    if (lane == 0) out[0] = start;
    for (int base = 0; base < count; base += 64) {
        const double mine = (base + lane < count) ? x[base + lane] : 0.0;
        double res = 0.0;
#pragma unroll
        for (int j = 0; j < 64; ++j) {
            acc = acc + __shfl(mine, j);
            if (lane == j) res = acc;
        }
        if (base + lane < count) out[base + lane + 1] = res;
    }
}
#pragma clang fp contract(fast)

// e^{-y} for y >= 0 with a 32-entry table: y = k ln2/32 + r, |r| <= ln2/64, e^{-y} =
// 2^-(k>>5) * tab[k&31] * e^{-r} with tab[j] = 2^(-j/32) and a degree-5 polynomial (error < 3e-15 + 1.2e-16 y:
// the reduction is one fused multiply-add with the double nearest to ln2/32, whose own error times k is all
// that is lost; beyond y = 40 the result is below 1e-17 of anything it is added to).
__device__ __forceinline__ double exp_neg(double y, const double* tab) {
    const double yc = fmin(y, 1000.0);
    const double kf = rint(yc * 46.166241308446828);
    const int ki = static_cast<int>(kf);
    const double tv = tab[ki & 31];
    const double r = -fma(kf, -(6.93147180559945309417e-01 / 32.0), yc);
    double p = 8.33333333333333333333e-03;
    p = fma(p, r, 4.16666666666666666667e-02);
    p = fma(p, r, 1.66666666666666666667e-01);
    p = fma(p, r, 0.5);
    p = fma(p, r, 1.0);
    p = fma(p, r, 1.0);
    return ldexp(p * tv, -(ki >> 5));                          // 2^-1442 flushes to 0
}

// Two of them at once, so that both table entries are on their way before either polynomial starts (the table read
// is the one long latency of the routine).
__device__ __forceinline__ void exp_neg2(double y0, double y1, const double* tab, double& x0, double& x1) {
    const double c0 = fmin(y0, 1000.0), c1 = fmin(y1, 1000.0);
    const double k0 = rint(c0 * 46.166241308446828), k1 = rint(c1 * 46.166241308446828);
    const int i0 = static_cast<int>(k0), i1 = static_cast<int>(k1);
    const double t0 = tab[i0 & 31], t1 = tab[i1 & 31];
    const double r0 = -fma(k0, -(6.93147180559945309417e-01 / 32.0), c0), r1 = -fma(k1, -(6.93147180559945309417e-01 / 32.0), c1);
    double p0 = 8.33333333333333333333e-03, p1 = 8.33333333333333333333e-03;
    p0 = fma(p0, r0, 4.16666666666666666667e-02); p1 = fma(p1, r1, 4.16666666666666666667e-02);
    p0 = fma(p0, r0, 1.66666666666666666667e-01); p1 = fma(p1, r1, 1.66666666666666666667e-01);
    p0 = fma(p0, r0, 0.5); p1 = fma(p1, r1, 0.5);
    p0 = fma(p0, r0, 1.0); p1 = fma(p1, r1, 1.0);
    p0 = fma(p0, r0, 1.0); p1 = fma(p1, r1, 1.0);
    x0 = ldexp(p0 * t0, -(i0 >> 5)); x1 = ldexp(p1 * t1, -(i1 >> 5));
}

// Candidate key: larger q first, ties to the lower token id.  q >= 0, so its bit pattern is
// monotone; the low word holds ~id so that a plain 64-bit compare gives the order.
__device__ __forceinline__ unsigned long long make_key(float q, int id) {
    return (static_cast<unsigned long long>(__float_as_uint(q)) << 32) |
           static_cast<unsigned long long>(0xFFFFFFFFu - static_cast<unsigned>(id));
}
// The same for a draft logit (any finite float): its bit pattern made monotone over the whole line.
__device__ __forceinline__ unsigned long long make_key_logit(float d, int id) {
    const unsigned b = __float_as_uint(d);
    const unsigned mono = (b & 0x80000000u) ? ~b : (b | 0x80000000u);
    return (static_cast<unsigned long long>(mono) << 32) | static_cast<unsigned long long>(0xFFFFFFFFu - static_cast<unsigned>(id));
}
// A double as a 64-bit pattern that rises with it (any finite value or infinity).
__device__ __forceinline__ unsigned long long mono64(double x) {
    const unsigned long long b = static_cast<unsigned long long>(__double_as_longlong(x));
    return (b >> 63) ? ~b : (b | 0x8000000000000000ull);
}
__device__ __forceinline__ unsigned mono32(float x) {
    const unsigned b = __float_as_uint(x);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
// The value whose decreasing order is that of q/p for rows given as logits: q/p is proportional to
// exp(d / Td - t / Tt).  With one temperature that is the order of d - t, exact in float64 for float32 logits; with
// two, the two products are rounded and then subtracted (no fused operation: the checker does the same three steps).
__device__ __forceinline__ double logit_ratio_key(double d, double t, double inv_td, double inv_tt) {
    return inv_td == inv_tt ? d - t : __dsub_rn(__dmul_rn(d, inv_td), __dmul_rn(t, inv_tt));
}
__device__ __forceinline__ float key_logit(unsigned long long key) {
    const unsigned mono = static_cast<unsigned>(key >> 32);
    return __uint_as_float((mono & 0x80000000u) ? (mono & 0x7FFFFFFFu) : ~mono);
}
__device__ __forceinline__ int key_id(unsigned long long key) {
    return static_cast<int>(0xFFFFFFFFu - static_cast<unsigned>(key & 0xFFFFFFFFull));
}
__device__ __forceinline__ float key_q(unsigned long long key) {
    return __uint_as_float(static_cast<unsigned>(key >> 32));
}

// A threshold theta such that exactly k of the `count` distinct keys held in LDS are >= theta
// (1 <= k <= count <= kSelCap; theta <= the k-th largest key), by most-significant-digit radix
// selection, 8 bits per pass.  The walk stops as soon as the bucket it enters holds exactly the keys
// still needed: theta is then that bucket's prefix with the lower digits zero.  All NT threads of the
// workgroup call it.  hist: LDS int[256]; pick: LDS int[4].
template <int NT = kThreads>
__device__ inline unsigned long long block_kth_largest(const unsigned long long* keys, int count, int k,
                                                       int* hist, int* pick) {
    const int tid = threadIdx.x;
    unsigned long long prefix = 0;
    int need = k;
    for (int shift = 56; shift >= 0; shift -= 8) {
        if (tid < 256) hist[tid] = 0;
        __syncthreads();
        const unsigned long long mask = (shift == 56) ? 0ull : (~0ull << (shift + 8));
        for (int i = tid; i < count; i += NT) {
            const unsigned long long key = keys[i];
            if ((key & mask) == prefix) atomicAdd(&hist[static_cast<int>((key >> shift) & 255ull)], 1);
        }
        __syncthreads();
        if (tid < 64) {
            // lane l owns digits 255-4l .. 252-4l (largest digits in lane 0)
            int c[4]; int tot = 0;
            for (int j = 0; j < 4; ++j) { c[j] = hist[255 - 4 * tid - j]; tot += c[j]; }
            int incl = tot;
            for (int o = 1; o < 64; o <<= 1) {
                int up = __shfl_up(incl, o);
                if (tid >= o) incl += up;
            }
            int excl = incl - tot;
            if (excl < need && need <= incl) {
                int above = excl;
                for (int j = 0; j < 4; ++j) {
                    if (need <= above + c[j]) { pick[0] = 255 - 4 * tid - j; pick[1] = need - above; pick[2] = c[j]; break; }
                    above += c[j];
                }
            }
        }
        __syncthreads();
        prefix |= static_cast<unsigned long long>(pick[0]) << shift;
        need = pick[1];
        const bool whole_bucket = pick[2] == need;
        __syncthreads();
        if (whole_bucket) break;
    }
    return prefix;
}

}  // namespace gr
