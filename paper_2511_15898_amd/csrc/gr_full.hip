// Full-vocabulary support: steps 1 and 2 of the verifier (Sec. 5.1 ratio order and prefix psi, Sec. 6
// H*, alpha*, outer residuals of Thm 6.2, records, truncation sets of Alg. 1) for a draft distribution
// without top-k or with a top-k above GR_MAX_SUPPORT, where the support (up to V tokens) does not fit LDS.
//
// Every per-token array lives in a per-handle HBM workspace, row-major with stride V + 2; one
// 256-thread workgroup works through a row.  The arithmetic that decides integers (prefix sums, F,
// the running masses of the truncation sets) is the same sequential fp64 arithmetic as on the
// LDS-resident path.
#include "gr_internal.h"

namespace gr {

namespace {

constexpr int kSortItems = 4;                      // keys per thread and tile
constexpr int kSortWaves = kSortItems * kWaves;    // 64-key groups of one tile, in index order

struct SortLds {
    int hist[8][256];                              // digit histograms of all eight passes
    int base[2][256];                              // first output slot of each digit for the current tile
    unsigned short wcnt[2][kSortWaves][256];       // per 64-key group: keys with this digit, then their offset within the tile
    int skip[8];
};

// Stable least-significant-digit radix sort of `count` (key, value) pairs of one row, ascending in the
// 64-bit key, 8 bits per pass, between the buffer pairs (k0, v0) and (k1, v1).  Returns 0 or 1: the pair
// that holds the result.  The histograms of all passes come from one read of the keys (they do not depend
// on the order); passes whose digit is the same for every key are skipped.  A pass moves tiles of 1024
// keys, four per thread, with two barriers per tile: the per-group counters and the digit bases are
// double-buffered, and thread d carries the running base of digit d in a register.  All threads call.
__device__ int block_radix_sort(unsigned long long* k0, int* v0, unsigned long long* k1, int* v1, int count,
                                SortLds& S) {
    constexpr int kTile = kThreads * kSortItems;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    for (int j = 0; j < 8; ++j) S.hist[j][tid] = 0;
    if (tid < 8) S.skip[tid] = 0;
    __syncthreads();
    for (int i0 = 0; i0 < count; i0 += kThreads) {
        const int i = i0 + tid;
        const bool valid = i < count;
        const unsigned long long key = valid ? k0[i] : 0ull;
        const unsigned long long vm = __ballot(valid);
        if (vm == 0ull) continue;                               // wave-uniform; lane 0 is valid otherwise
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int d = static_cast<int>((key >> (8 * j)) & 255ull);
            const int d0 = __builtin_amdgcn_readfirstlane(d);
            if (__ballot(valid && d == d0) == vm) {             // one digit in the whole wave: one update
                if (lane == 0) atomicAdd(&S.hist[j][d0], __popcll(vm));
            } else if (valid) {
                atomicAdd(&S.hist[j][d], 1);
            }
        }
    }
    __syncthreads();
    for (int j = 0; j < 8; ++j) if (S.hist[j][tid] == count) S.skip[j] = 1;
    __syncthreads();

    int cur = 0;
    for (int pass = 0; pass < 8; ++pass) {
        if (S.skip[pass]) continue;
        const int shift = 8 * pass;
        const unsigned long long* ks = cur ? k1 : k0; const int* vs = cur ? v1 : v0;
        unsigned long long* kd = cur ? k0 : k1; int* vd = cur ? v0 : v1;
        if (wv == 0) {
            // exclusive scan of the histogram: lane l owns digits 4l .. 4l+3; the result goes to base[1]
            // (unused until the second tile) and from there to the owners' registers
            int c[4]; int tot = 0;
            for (int j = 0; j < 4; ++j) { c[j] = S.hist[pass][4 * lane + j]; tot += c[j]; }
            int incl = tot;
            for (int o = 1; o < 64; o <<= 1) { const int up = __shfl_up(incl, o); if (lane >= o) incl += up; }
            int run = incl - tot;
            for (int j = 0; j < 4; ++j) { S.base[1][4 * lane + j] = run; run += c[j]; }
        }
        for (int w = 0; w < kSortWaves; ++w) { S.wcnt[0][w][tid] = 0; S.wcnt[1][w][tid] = 0; }
        __syncthreads();
        int mybase = S.base[1][tid];                            // running first slot of digit `tid`
        __syncthreads();
        unsigned long long kn[kSortItems]; int vn[kSortItems];
#pragma unroll
        for (int j = 0; j < kSortItems; ++j) {
            const int i = j * kThreads + tid;
            kn[j] = 0ull; vn[j] = 0;
            if (i < count) { kn[j] = ks[i]; vn[j] = vs[i]; }
        }
        int buf = 0;
        for (int t0 = 0; t0 < count; t0 += kTile, buf ^= 1) {
            unsigned long long key[kSortItems]; int val[kSortItems]; int dig[kSortItems]; int rank[kSortItems];
#pragma unroll
            for (int j = 0; j < kSortItems; ++j) { key[j] = kn[j]; val[j] = vn[j]; }
#pragma unroll
            for (int j = 0; j < kSortItems; ++j) {
                const int i = t0 + kTile + j * kThreads + tid;
                if (i < count) { kn[j] = ks[i]; vn[j] = vs[i]; }
            }
#pragma unroll
            for (int j = 0; j < kSortItems; ++j) {
                const bool valid = t0 + j * kThreads + tid < count;
                const int d = static_cast<int>((key[j] >> shift) & 255ull);
                // lanes of this wave that hold the same digit
                unsigned long long peers = __ballot(valid);
#pragma unroll
                for (int b = 0; b < 8; ++b) {
                    const bool bit = (d >> b) & 1;
                    const unsigned long long m = __ballot(valid && bit);
                    peers &= bit ? m : ~m;
                }
                dig[j] = d;
                rank[j] = __popcll(peers & ((1ull << lane) - 1ull));
                if (valid && rank[j] == 0) S.wcnt[buf][j * kWaves + wv][d] = static_cast<unsigned short>(__popcll(peers));
            }
            __syncthreads();
            {
                // digit `tid`: counts of the groups -> offsets within the tile; clear the other buffer for the next tile
                S.base[buf][tid] = mybase;
                int run = 0;
#pragma unroll
                for (int w = 0; w < kSortWaves; ++w) {
                    const int c = S.wcnt[buf][w][tid];
                    S.wcnt[buf][w][tid] = static_cast<unsigned short>(run);
                    run += c;
                    S.wcnt[buf ^ 1][w][tid] = 0;
                }
                mybase += run;
            }
            __syncthreads();
#pragma unroll
            for (int j = 0; j < kSortItems; ++j) {
                if (t0 + j * kThreads + tid < count) {
                    const int off = S.base[buf][dig[j]] + S.wcnt[buf][j * kWaves + wv][dig[j]] + rank[j];
                    kd[off] = key[j]; vd[off] = val[j];
                }
            }
        }
        cur ^= 1;
        __syncthreads();
    }
    return cur;
}

#pragma clang fp contract(off)
// The running sums of wave_sequential_scan for operands in LDS: every lane reads x[j] (one address
// for the whole wave: a broadcast read) and adds it, so all lanes hold the same sums, in the order of
// a sequential loop; lane 0 stores them.  x must be readable and zero, out writable, up to the next
// multiple of 64 beyond `count`.  out[0] = start, out[i + 1] = start + x[0] + ... + x[i].
__device__ __forceinline__ void wave_sequential_scan_padded(const double* x, double* out, int count, double start) {
    const int lane = threadIdx.x & 63;
    double acc = start;
    if (lane == 0) out[0] = start;
    for (int base = 0; base < count; base += 64) {
        double a[64];
#pragma unroll
        for (int j = 0; j < 64; ++j) { acc = acc + x[base + j]; a[j] = acc; }
        if (lane == 0) {
#pragma unroll
            for (int j = 0; j < 64; ++j) out[base + j + 1] = a[j];
        }
    }
}
#pragma clang fp contract(fast)

// Exclusive suffix minimum over the 256 threads: min of v over the threads after this one (1e300 for
// the last); *total = min over all.  buf0, buf1: LDS double[256].
__device__ double block_suffix_min_excl(double v, double* buf0, double* buf1, double* total) {
    const int tid = threadIdx.x;
    double* src = buf0; double* dst = buf1;
    src[tid] = v;
    __syncthreads();
    for (int o = 1; o < kThreads; o <<= 1) {
        dst[tid] = (tid + o < kThreads) ? fmin(src[tid], src[tid + o]) : src[tid];
        __syncthreads();
        double* t = src; src = dst; dst = t;
    }
    const double excl = (tid + 1 < kThreads) ? src[tid + 1] : 1e300;
    *total = src[0];
    __syncthreads();
    return excl;
}

// Exclusive prefix sum over the 256 threads; *total = sum over all.  buf0, buf1: LDS int[256].
__device__ int block_prefix_sum_excl(int v, int* buf0, int* buf1, int* total) {
    const int tid = threadIdx.x;
    int* src = buf0; int* dst = buf1;
    src[tid] = v;
    __syncthreads();
    for (int o = 1; o < kThreads; o <<= 1) {
        dst[tid] = (tid >= o) ? src[tid] + src[tid - o] : src[tid];
        __syncthreads();
        int* t = src; src = dst; dst = t;
    }
    const int excl = src[tid] - v;
    *total = src[kThreads - 1];
    __syncthreads();
    return excl;
}

// chist[4096]: members per magnitude class of a positive float (its bit pattern >> 19: exponent and four mantissa
// bits; every member lies below the class's upper edge, so count x edge bounds the class's mass).  Classes are
// dropped from the bottom while that bound stays within `budget`; returns the lowest class that stays (0 when every
// class would fit: nothing is dropped then).  dscan: LDS double[kThreads], bsel: LDS int.  All threads call.
__device__ int class_threshold(const int* chist, double budget, double* dscan, int* bsel) {
    const int tid = threadIdx.x;
    // thread t owns classes 16 t .. 16 t + 15; prefix of the bounds over the threads, serially by thread 0
    double local = 0.0;
    for (int c = 16 * tid; c < 16 * tid + 16; ++c)
        local += static_cast<double>(chist[c]) * static_cast<double>(__uint_as_float((static_cast<unsigned>(c) + 1u) << 19));
    dscan[tid] = local;
    if (tid == 0) *bsel = 4096;
    __syncthreads();
    if (tid == 0) { double run = 0.0; for (int t = 0; t < kThreads; ++t) { const double v = dscan[t]; dscan[t] = run; run += v; } }
    __syncthreads();
    {
        double run = dscan[tid];                                 // bound on the mass of all classes below 16 tid
        for (int c = 16 * tid; c < 16 * tid + 16; ++c) {
            run += static_cast<double>(chist[c]) * static_cast<double>(__uint_as_float((static_cast<unsigned>(c) + 1u) << 19));
            if (run > budget) { atomicMin(bsel, c); break; }     // class c cannot be dropped whole
        }
    }
    __syncthreads();
    const int b = *bsel;
    __syncthreads();
    return b == 4096 ? 0 : b;
}

__device__ void mark_bad(const FullParams& fp, int row, double ptot, double qtot) {
    RowInfo info;
    info.support = 0; info.h = 0; info.status = GR_ROW_BAD; info.iterations = 0;
    info.alpha_star = __longlong_as_double(0x7ff8000000000000ll);
    info.res_total = 0.0; info.p_total = ptot; info.q_total = qtot; info.node_tokens = 0.0; info.p_ref = 0.0; info.inv_temp = 0.0; info.q_ref = 0.0;
    fp.info[row] = info;
    fp.accept_prob[row] = __uint_as_float(0x7fc00000u);
    fp.status[row] = GR_ROW_BAD;
}

}  // namespace

// ---- kernel 1: row sums and validity, the support (all positive entries of q, or the k largest) in
// token order, sort by decreasing q/p (ties by id).
// The sort key is the correctly rounded float64 quotient q/p: for float32 inputs two different
// ratios differ by at least 2^-48 relative, so their quotients differ and keep their order, and equal
// ratios give equal quotients -- the same order as the exact cross-product comparison (Sec. 5.1).
__global__ __launch_bounds__(kThreads) void full_order_kernel(FullParams fp) {
    __shared__ SortLds S;
    __shared__ double red[kWaves];
    __shared__ int wtot[4 * kWaves];
    __shared__ double dscan[kThreads];
    __shared__ double xin[kThreads];
    __shared__ double xout[kThreads + 1];
    __shared__ int bsel;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, row = blockIdx.x;
    const int V = fp.V;
    const size_t vs = static_cast<size_t>(V) + 2;
    const float* pr = fp.p + static_cast<size_t>(row) * V;
    const float* qr = fp.q + static_cast<size_t>(row) * V;
    unsigned long long* k0 = fp.key0 + row * vs; unsigned long long* k1 = fp.key1 + row * vs;
    int* v0 = fp.val0 + row * vs; int* v1 = fp.val1 + row * vs;

    double ptot, qtot;
    double p_ref = 0.0, q_ref = 0.0, inv_temp = 0.0, inv_temp_q = 0.0;
    if (fp.logits) {
        // rows given as logits: the largest target and draft logit, then the target's softmax sum relative to it;
        // q needs no sum (it is renormalised over the support).  A NaN or +inf anywhere, or a temperature that is not
        // positive and finite, marks the row bad; -inf is a masked token.
        const float T = fp.temperature[row];
        const float Td = fp.draft_temperature ? fp.draft_temperature[row] : T;
        float tm = -__builtin_inff(), dm = -__builtin_inff(); int bad = !(T > 0.f) || !(T <= 3.0e38f) || !(Td > 0.f) || !(Td <= 3.0e38f);
        for (int i = tid; i < V; i += kThreads) {
            const float pv = pr[i], qv = qr[i];
            bad |= !(pv + qv < 3.0e38f);
            tm = fmaxf(tm, pv); dm = fmaxf(dm, qv);
        }
        p_ref = block_max(static_cast<double>(tm), red);
        q_ref = block_max(static_cast<double>(dm), red);
        const int anybad = block_sum_i(bad, red);
        inv_temp = anybad ? 0.0 : 1.0 / static_cast<double>(T);
        inv_temp_q = anybad ? 0.0 : 1.0 / static_cast<double>(Td);
        double ps = 0.0;
        if (!anybad && p_ref > -3.0e38 && q_ref > -3.0e38)
            for (int i = tid; i < V; i += kThreads) ps += exp((static_cast<double>(pr[i]) - p_ref) * inv_temp);
        ptot = block_sum(ps, red); qtot = 1.0;
        if (anybad || !(ptot >= 1.0) || !(ptot < 1e300)) {
            if (tid == 0) mark_bad(fp, row, ptot, qtot);
            return;
        }
    } else {
        double ps = 0.0, qs = 0.0; int bad = 0;
        for (int i = tid; i < V; i += kThreads) {
            const float pv = pr[i], qv = qr[i];
            bad |= !(qv >= 0.f) | !(pv >= 0.f);
            ps += static_cast<double>(pv); qs += static_cast<double>(qv);
        }
        ptot = block_sum(ps, red);
        qtot = block_sum(qs, red);
        const int anybad = block_sum_i(bad, red);
        if (anybad || !(fabs(ptot - 1.0) <= 1e-3) || !(fabs(qtot - 1.0) <= 1e-3)) {
            if (tid == 0) mark_bad(fp, row, ptot, qtot);
            return;
        }
    }
    const bool lg = fp.logits != 0;
    // With a top-k below the number of positive entries, or a nucleus cut (tail_mass > 0; Sec. 5.1: top-p/k
    // sampling of the draft restricts the domain): order the candidates by decreasing q (ties by token id)
    // and flag the first k' of them; the support is then the flagged tokens.
    int* member = fp.flag + row * vs;                       // by token id here; reused by rank later
    bool by_flag = false;
    const bool cut = fp.tail_mass > 0.0;
    if (fp.k < V || cut) {
        // Nucleus cut: tokens are taken by decreasing q until their running sum reaches (1 - tail_mass) qtot.
        // Candidates first, so that only they are sorted: half of the budget tail_mass qtot goes to the tokens
        // below qmin = budget / (2 V) (fewer than V of them: below budget / 2 together), the other half to the
        // lowest occupied magnitude classes (exponent and four mantissa bits of q: every member is below the
        // class's upper edge, so count x edge bounds the class's mass).  Everything dropped here lies in the
        // tail that the exact walk below would leave out anyway.
        double qmin = 0.0; int bstar = 0;
        if (cut) {
            int* chist = reinterpret_cast<int*>(&S.wcnt[0][0][0]);          // 4096 classes = the sort's 16 KB of counters
            static_assert(sizeof(S.wcnt) >= 4096 * sizeof(int), "the class histogram borrows the sort's counters");
            for (int c = tid; c < 4096; c += kThreads) chist[c] = 0;
            __syncthreads();
            const double budget = fp.tail_mass * qtot;
            qmin = 0.5 * budget / static_cast<double>(V);
            for (int i = tid; i < V; i += kThreads) {
                const float qv = qr[i];
                if (static_cast<double>(qv) >= qmin && qv > 0.f) atomicAdd(&chist[__float_as_uint(qv) >> 19], 1);
            }
            __syncthreads();
            bstar = class_threshold(chist, 0.5 * budget, dscan, &bsel);
        }
        int cnt = 0;
        for (int t0 = 0; t0 < V; t0 += 4 * kThreads) {           // 1024 tokens per round
            float qv[4]; unsigned long long mask[4]; bool take[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) { const int i = t0 + j * kThreads + tid; qv[j] = i < V ? qr[i] : (lg ? -__builtin_inff() : 0.f); }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                take[j] = (lg ? qv[j] > -3.0e38f : qv[j] > 0.f) && (!cut || (static_cast<double>(qv[j]) >= qmin && static_cast<int>(__float_as_uint(qv[j]) >> 19) >= bstar));
                mask[j] = __ballot(take[j]);
                if (lane == 0) wtot[j * kWaves + wv] = __popcll(mask[j]);
            }
            __syncthreads();
            int run = 0, offs[4] = {0, 0, 0, 0};
#pragma unroll
            for (int g = 0; g < 4 * kWaves; ++g) {
#pragma unroll
                for (int j = 0; j < 4; ++j) if (g == j * kWaves + wv) offs[j] = run;
                run += wtot[g];
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int i = t0 + j * kThreads + tid;
                if (take[j]) {
                    const int off = cnt + offs[j] + __popcll(mask[j] & ((1ull << lane) - 1ull));
                    k0[off] = static_cast<unsigned long long>(lg ? ~mono32(qv[j]) : ~__float_as_uint(qv[j]));   // ties: the sort is stable and this is token order
                    v0[off] = i;
                }
                if (i < V) member[i] = 0;
            }
            cnt += run;
            __syncthreads();
        }
        if (cnt > fp.k || (cut && cnt > 0)) {
            const int res = block_radix_sort(k0, v0, k1, v1, cnt, S);
            const int* sorted = res ? v1 : v0;
            int keep = cnt;
            if (cut) {
                // the exact walk: running sums of q in the sorted order, added one after the other (wave 0), until
                // they reach (1 - tail_mass) qtot; the first rank that does is the last token of the support
                const double need = (1.0 - fp.tail_mass) * qtot;
                double carry = 0.0;
                if (tid == 0) bsel = cnt;                                // rank of the last kept token; cnt: never reached
                __syncthreads();
                for (int t0 = 0; t0 < cnt; t0 += kThreads) {
                    const int r = t0 + tid;
                    xin[tid] = r < cnt ? static_cast<double>(qr[sorted[r]]) : 0.0;
                    __syncthreads();
                    if (wv == 0) wave_sequential_scan_padded(xin, xout, kThreads, carry);
                    __syncthreads();
                    if (r < cnt && xout[tid + 1] >= need) atomicMin(&bsel, r);
                    carry = xout[kThreads];
                    __syncthreads();
                    if (bsel < cnt) break;                               // uniform: read behind the barrier
                }
                keep = bsel < cnt ? bsel + 1 : cnt;
                __syncthreads();
            }
            if (fp.k < keep) keep = fp.k;
            for (int r = tid; r < keep; r += kThreads) member[sorted[r]] = 1;
            by_flag = true;
        }
        __syncthreads();
    }
    // the support in token order, with its keys
    int kk = 0;
    for (int t0 = 0; t0 < V; t0 += 4 * kThreads) {               // 1024 tokens per round
        float qv[4], pv[4]; bool in[4]; unsigned long long mask[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int i = t0 + j * kThreads + tid;
            qv[j] = i < V ? qr[i] : (lg ? -__builtin_inff() : 0.f); pv[j] = i < V ? pr[i] : 1.f;
            in[j] = by_flag ? (i < V && member[i] != 0) : (lg ? qv[j] > -3.0e38f : qv[j] > 0.f);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            mask[j] = __ballot(in[j]);
            if (lane == 0) wtot[j * kWaves + wv] = __popcll(mask[j]);
        }
        __syncthreads();
        int run = 0, offs[4] = {0, 0, 0, 0};
#pragma unroll
        for (int g = 0; g < 4 * kWaves; ++g) {
#pragma unroll
            for (int j = 0; j < 4; ++j) if (g == j * kWaves + wv) offs[j] = run;
            run += wtot[g];
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (in[j]) {
                const int off = kk + offs[j] + __popcll(mask[j] & ((1ull << lane) - 1ull));
                // rows given as logits: q/p is proportional to exp((d - t) / T), so the order is that of d - t (exact in
                // float64 for float32 logits; a masked target gives +inf: first)
                const double ratio = lg ? logit_ratio_key(static_cast<double>(qv[j]), static_cast<double>(pv[j]), inv_temp_q, inv_temp)
                                        : static_cast<double>(qv[j]) / static_cast<double>(pv[j]);   // p = 0 gives +inf: first
                k0[off] = lg ? ~mono64(ratio) : ~static_cast<unsigned long long>(__double_as_longlong(ratio));
                v0[off] = t0 + j * kThreads + tid;
            }
        }
        kk += run;
        __syncthreads();
    }
    if (kk == 0) {
        if (tid == 0) mark_bad(fp, row, ptot, qtot);
        return;
    }
    __syncthreads();
    const int res = block_radix_sort(k0, v0, k1, v1, kk, S);
    const int* sorted = res ? v1 : v0;
    int* order = fp.order + row * vs;
    for (int r = tid; r < kk; r += kThreads) order[r] = sorted[r];
    if (tid == 0) {
        RowInfo info;
        info.support = kk; info.h = 0; info.status = GR_ROW_OK; info.iterations = 0;
        info.alpha_star = 0.0; info.res_total = 0.0; info.p_total = ptot; info.q_total = qtot; info.node_tokens = 0.0;
        info.p_ref = p_ref; info.inv_temp = inv_temp; info.q_ref = q_ref;
        fp.info[row] = info;
    }
}

// ---- kernel 2: prefix sums in the order, F, H*, alpha*, suffix minima, residuals, records, blocks.
__global__ __launch_bounds__(kThreads) void full_scan_kernel(FullParams fp) {
    constexpr int kTile = 1024;
    __shared__ double xin[2][kTile];
    __shared__ double xout[2][kTile + 1];
    __shared__ double red[kWaves];
    __shared__ double dbuf[2][kThreads];
    __shared__ int ibuf[2][kThreads];
    const int tid = threadIdx.x, wv = tid >> 6, row = blockIdx.x;
    const int V = fp.V, n = fp.n;
    const size_t vs = static_cast<size_t>(V) + 2;
    RowInfo info = fp.info[row];
    if (info.status == GR_ROW_BAD) return;
    const int kk = info.support;
    const double inv_temp_q = fp.logits ? 1.0 / static_cast<double>(fp.draft_temperature ? fp.draft_temperature[row] : fp.temperature[row]) : 0.0;
    const float* pr = fp.p + static_cast<size_t>(row) * V;
    const float* qr = fp.q + static_cast<size_t>(row) * V;
    const int* order = fp.order + row * vs;
    double* pn = fp.pn + row * vs; double* qn = fp.qn + row * vs;
    double* P = fp.P + row * vs; double* Q = fp.Q + row * vs; double* F = fp.F + row * vs;
    double* rho = fp.rho + row * vs; double* tgt = fp.tgt + row * vs;
    int* flag = fp.flag + row * vs; int* blk = fp.blk + row * vs; int* blo = fp.blo + row * vs;
    int* inT = fp.inT + row * vs; int* bcount = fp.bcount + row * vs;

    for (int r0 = tid; r0 < kk; r0 += 4 * kThreads) {           // four independent gathers per thread in flight
        int id[4]; float pv[4], qv[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) { const int r = r0 + j * kThreads; id[j] = r < kk ? order[r] : 0; }
#pragma unroll
        for (int j = 0; j < 4; ++j) { pv[j] = pr[id[j]]; qv[j] = qr[id[j]]; }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int r = r0 + j * kThreads;
            if (r < kk) {
                if (fp.logits) {
                    pn[r] = exp((static_cast<double>(pv[j]) - info.p_ref) * info.inv_temp) / info.p_total;
                    qn[r] = exp((static_cast<double>(qv[j]) - info.q_ref) * inv_temp_q);
                } else {
                    pn[r] = static_cast<double>(pv[j]) / info.p_total;
                    qn[r] = static_cast<double>(qv[j]);          // raw q for now
                }
                inT[r] = 0;
            }
        }
    }
    if (tid == 0) { P[0] = 0.0; Q[0] = 0.0; }
    __syncthreads();
    // sequential prefix sums, a tile at a time through LDS (wave 0: p, wave 1: q); the next tile is
    // loaded into registers while the two waves scan
    double carry_p = 0.0, carry_q = 0.0;
    double np_[4], nq_[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int i = j * kThreads + tid;
        np_[j] = i < kk ? pn[i] : 0.0; nq_[j] = i < kk ? qn[i] : 0.0;
    }
    for (int t0 = 0; t0 < kk; t0 += kTile) {
        const int cnt = min(kTile, kk - t0);
#pragma unroll
        for (int j = 0; j < 4; ++j) { xin[0][j * kThreads + tid] = np_[j]; xin[1][j * kThreads + tid] = nq_[j]; }   // zeros beyond cnt
        __syncthreads();
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int i = t0 + kTile + j * kThreads + tid;
            np_[j] = i < kk ? pn[i] : 0.0; nq_[j] = i < kk ? qn[i] : 0.0;
        }
        if (wv == 0) wave_sequential_scan_padded(xin[0], xout[0], cnt, carry_p);
        if (wv == 1) wave_sequential_scan_padded(xin[1], xout[1], cnt, carry_q);
        __syncthreads();
        for (int i = tid; i < cnt; i += kThreads) { P[t0 + i + 1] = xout[0][i + 1]; Q[t0 + i + 1] = xout[1][i + 1]; }
        carry_p = xout[0][cnt]; carry_q = xout[1][cnt];
        // the next tile's scan, which overwrites xout, starts behind the next barrier
    }
    __syncthreads();                                            // P and Q are read back below by other threads than wrote them
    const double stot = carry_q;
    double fmin_local = 1e300, hcand = 1e18;                    // this thread's smallest F and the first rank that has it
    {
#pragma clang fp contract(off)
        for (int m0 = tid; m0 <= kk; m0 += 4 * kThreads) {
            double Qv[4], Pv[4], qv[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int m = m0 + j * kThreads;
                Qv[j] = m <= kk ? Q[m] : 0.0; Pv[j] = m <= kk ? P[m] : 0.0; qv[j] = m < kk ? qn[m] : 0.0;
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int m = m0 + j * kThreads;
                if (m <= kk) {
                    const double Qm = Qv[j] / stot;
                    Q[m] = Qm;
                    const double Fm = (m == 0) ? 0.0 : Pv[j] - ipow(Qm, n);
                    F[m] = Fm;
                    if (Fm < fmin_local) { fmin_local = Fm; hcand = static_cast<double>(m); }   // ranks rise within a thread
                    if (m < kk) qn[m] = qv[j] / stot;
                }
            }
        }
    }
    __syncthreads();
    // H*: the smallest minimising prefix
    const double Fmin = block_min(fmin_local, red);
    const int h = static_cast<int>(block_min(fmin_local == Fmin ? hcand : 1e18, red));
    // G = suffix minima of F over m = 0..kk, tiles of 1024 from the top down (4 consecutive entries per
    // thread); G is only needed here, so residuals, targets and records (F(m) <= G(m+1) for m >= h;
    // m = kk always) are taken in the same sweep and G is never stored
    {
        double later = 1e300;                                   // min of F over the tiles above
        const int ntile = (kk + 1 + kTile - 1) / kTile;
        for (int t = ntile - 1; t >= 0; --t) {
            const int m0 = t * kTile + tid * 4;
            double a[4], pv[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) { a[j] = (m0 + j <= kk) ? F[m0 + j] : 1e300; pv[j] = (m0 + j < kk) ? pn[m0 + j] : 0.0; }
            double s[4];
            s[3] = a[3]; s[2] = fmin(a[2], s[3]); s[1] = fmin(a[1], s[2]); s[0] = fmin(a[0], s[1]);
            double total;
            const double after = fmin(block_suffix_min_excl(s[0], dbuf[0], dbuf[1], &total), later);   // G(m0 + 4)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int m = m0 + j;
                if (m <= kk) {
                    const double g = fmin(s[j], after);                                  // G(m)
                    const double gn = (j < 3) ? fmin(s[j + 1], after) : after;           // G(m + 1), unused at m = kk
                    flag[m] = (m >= h && (m == kk || a[j] <= gn)) ? 1 : 0;
                    if (m < kk) {
                        const double r = (m >= h) ? gn - g : 0.0;
                        rho[m] = r; tgt[m] = pv[j] - r;
                    }
                }
            }
            later = fmin(later, total);
        }
    }
    __syncthreads();
    // inclusive count of records -> block of each token outside H*, record positions
    int nrec = 0;
    {
        const int ntile = (kk + 1 + kTile - 1) / kTile;
        for (int t = 0; t < ntile; ++t) {
            const int m0 = t * kTile + tid * 4;
            int f[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) f[j] = (m0 + j <= kk) ? flag[m0 + j] : 0;
            int total;
            int run = nrec + block_prefix_sum_excl(f[0] + f[1] + f[2] + f[3], ibuf[0], ibuf[1], &total);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int m = m0 + j;
                if (m <= kk) {
                    run += f[j];
                    if (f[j]) blo[run] = m;                     // record number `run` (1-based) sits at rank m
                    if (m < kk) blk[m] = (m >= h) ? run : 0;    // token m lies after record `run`
                }
            }
            nrec += total;
        }
    }
    __syncthreads();
    for (int b = tid; b <= nrec; b += kThreads) bcount[b] = 0;
    if (tid == 0) {
        info.h = h;
        info.alpha_star = 1.0 + F[h];
        info.res_total = -F[h];
        fp.info[row] = info;
        fp.nblk[row] = nrec - 1;
        fp.accept_prob[row] = static_cast<float>(1.0 + F[h]);
    }
}

// ---- kernel 3: truncation sets (Alg. 1: fewest tokens by decreasing q with gamma_T <= tau inside H*,
// epsilon_T <= tau outside), size of every program, row status.
__global__ __launch_bounds__(kThreads) void full_trunc_kernel(FullParams fp) {
    __shared__ SortLds S;
    __shared__ int cnt_in, cnt_out, act_in, capped, bsel;
    __shared__ int wtot[8 * kWaves];
    __shared__ double dscan[kThreads];
    __shared__ double wx[2][64];
    __shared__ double wo[2][65];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, row = blockIdx.x;
    const int V = fp.V, n = fp.n;
    const size_t vs = static_cast<size_t>(V) + 2;
    const RowInfo info = fp.info[row];
    if (info.status == GR_ROW_BAD) return;
    const int kk = info.support, h = info.h;
    const float* qr = fp.q + static_cast<size_t>(row) * V;
    const int* order = fp.order + row * vs;
    unsigned long long* k0 = fp.key0 + row * vs; unsigned long long* k1 = fp.key1 + row * vs;
    int* v0 = fp.val0 + row * vs; int* v1 = fp.val1 + row * vs;
    int* byq = fp.byq + row * vs;
    const double* qn = fp.qn + row * vs; const double* Q = fp.Q + row * vs; const double* tgt = fp.tgt + row * vs;
    const int* blk = fp.blk + row * vs; const int* blo = fp.blo + row * vs;
    int* inT = fp.inT + row * vs; int* bcount = fp.bcount + row * vs;

    // A token joins a truncation set only while the mass before it leaves more than tau.  The lowest-q tokens whose
    // normalised masses sum to at most tau / n can therefore never join: before any of them lies everything else of
    // its side, so what is left is at most Q^n - (Q - tau/n)^n <= tau.  They are left out of the sort (found, safely,
    // with the magnitude-class histogram: count x upper edge bounds a class's mass); the walk over the others is
    // the same arithmetic as before.
    int bstar = 0;
    if (fp.tau > 0.0) {
        int* chist = reinterpret_cast<int*>(&S.wcnt[0][0][0]);
        for (int c = tid; c < 4096; c += kThreads) chist[c] = 0;
        __syncthreads();
        for (int r = tid; r < kk; r += kThreads) {
            const float qf = static_cast<float>(qn[r]);
            if (qf > 0.f) atomicAdd(&chist[__float_as_uint(qf) >> 19], 1);
        }
        __syncthreads();
        bstar = class_threshold(chist, (fp.tau / static_cast<double>(n)) * (1.0 - 1e-6), dscan, &bsel);   // the margin covers the rounding of q to float
    }
    // ranks by (inside H* first, decreasing q, token id) of the tokens that stay, compacted in rank order
    int kept = 0, kept_in = 0;
    for (int t0 = 0; t0 < kk; t0 += 4 * kThreads) {               // 1024 ranks per round
        int id[4]; float qv[4]; bool take[4]; unsigned long long mask[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) { const int r = t0 + j * kThreads + tid; id[j] = r < kk ? order[r] : 0; }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int r = t0 + j * kThreads + tid;
            qv[j] = qr[id[j]];
            const float qf = r < kk ? static_cast<float>(qn[r]) : 0.f;
            take[j] = r < kk && (bstar == 0 || static_cast<int>(__float_as_uint(qf) >> 19) >= bstar);
            mask[j] = __ballot(take[j]);
            const unsigned long long in_mask = __ballot(take[j] && r < h);
            if (lane == 0) { wtot[j * kWaves + wv] = __popcll(mask[j]); wtot[4 * kWaves + j * kWaves + wv] = __popcll(in_mask); }
        }
        __syncthreads();
        int run = 0, run_in = 0, offs[4] = {0, 0, 0, 0};
#pragma unroll
        for (int g = 0; g < 4 * kWaves; ++g) {
#pragma unroll
            for (int j = 0; j < 4; ++j) if (g == j * kWaves + wv) offs[j] = run;
            run += wtot[g]; run_in += wtot[4 * kWaves + g];
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int r = t0 + j * kThreads + tid;
            if (take[j]) {
                const int off = kept + offs[j] + __popcll(mask[j] & ((1ull << lane) - 1ull));
                // q < 2, so bit 31 of ~bits(q) is always set: it carries the class instead (seven digits, not eight)
                // rows given as logits: decreasing q is decreasing draft logit, whose pattern needs all 32 bits; the class moves up
                const unsigned long long qb = fp.logits
                    ? (static_cast<unsigned long long>(~mono32(qv[j])) | (r < h ? 0ull : 0x100000000ull))
                    : static_cast<unsigned long long>((~__float_as_uint(qv[j]) & 0x7FFFFFFFu) | (r < h ? 0u : 0x80000000u));
                k0[off] = (qb << 24) | static_cast<unsigned long long>(id[j]);
                v0[off] = r;
            }
        }
        kept += run; kept_in += run_in;
        __syncthreads();
    }
    if (tid == 0) { cnt_in = 0; cnt_out = 0; act_in = 0; capped = 0; }
    __syncthreads();
    const int* sorted = v0;
    if (kept > 0) {
        const int res = block_radix_sort(k0, v0, k1, v1, kept, S);
        sorted = res ? v1 : v0;
    }
    for (int i = tid; i < kept; i += kThreads) byq[i] = sorted[i];
    __syncthreads();
    const double Qh = Q[h];
    // wave 0 walks H* by decreasing q, wave 1 the other tokens: a token joins T while the mass before
    // it leaves more than tau (running sums added one after the other, as a sequential loop would).
    // The walk only counts; the ranks and masses of the next two rounds are already on their way.
    if (wv < 2) {
#pragma clang fp contract(off)
        const int first = wv == 0 ? 0 : kept_in;                 // the tokens of H* that stayed come first
        const int len = wv == 0 ? kept_in : kept - kept_in;
        const double bound = wv == 0 ? ipow(Qh, n) : 1.0;
        double acc = wv == 0 ? 0.0 : Qh;
        int taken = 0;
        bool done = false;
        int r1 = (lane < len) ? byq[first + lane] : 0;                        // ranks of round 0
        int r2 = (64 + lane < len) ? byq[first + 64 + lane] : 0;              // ranks of round 1
        double m1 = (lane < len) ? qn[r1] : 0.0;                              // masses of round 0
        for (int base = 0; base < len && !done; base += 64) {
            const bool valid = base + lane < len;
            const double mine = m1;
            m1 = (base + 64 + lane < len) ? qn[r2] : 0.0;
            r2 = (base + 128 + lane < len) ? byq[first + base + 128 + lane] : 0;
            // running sums through a wave-private LDS strip (broadcast reads; see the padded scan)
            wx[wv][lane] = mine;
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront"); __builtin_amdgcn_wave_barrier();
            wave_sequential_scan_padded(wx[wv], wo[wv], 64, acc);
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront"); __builtin_amdgcn_wave_barrier();
            const double before = wo[wv][lane];
            acc = wo[wv][64];
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront"); __builtin_amdgcn_wave_barrier();
            const double bn = (before > 0.0) ? ipow(before, n) : 0.0;
            const bool in = valid && (bound - bn > fp.tau);
            const unsigned long long out_mask = __ballot(valid && !in);
            int upto = 64;                                       // lanes below `upto` join T
            if (out_mask) { upto = __ffsll(static_cast<long long>(out_mask)) - 1; done = true; }
            taken += __popcll(__ballot(valid && lane < upto));
        }
        if (lane == 0) { if (wv == 0) cnt_in = taken; else cnt_out = taken; }
    }
    __syncthreads();
    // mark the members of both sets; count the active ones per program
    {
        const int nin = cnt_in, nout = cnt_out;
        int act = 0;
        for (int i0 = tid; i0 < nin; i0 += 4 * kThreads) {
            int r[4]; double t[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) { const int i = i0 + j * kThreads; r[j] = i < nin ? byq[i] : -1; }
#pragma unroll
            for (int j = 0; j < 4; ++j) t[j] = r[j] >= 0 ? tgt[r[j]] : 0.0;
#pragma unroll
            for (int j = 0; j < 4; ++j) if (r[j] >= 0) { inT[r[j]] = 1; act += t[j] > 0.0; }
        }
        if (act) atomicAdd(&act_in, act);
        for (int i0 = tid; i0 < nout; i0 += 4 * kThreads) {
            int r[4]; double t[4]; int bl[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) { const int i = i0 + j * kThreads; r[j] = i < nout ? byq[kept_in + i] : -1; }
#pragma unroll
            for (int j = 0; j < 4; ++j) { t[j] = r[j] >= 0 ? tgt[r[j]] : 0.0; bl[j] = r[j] >= 0 ? blk[r[j]] : 0; }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (r[j] < 0) continue;
                inT[r[j]] = 1;
                if (t[j] > 0.0 && blo[bl[j] + 1] - blo[bl[j]] >= 2) {
                    const int old = atomicAdd(&bcount[bl[j]], 1);
                    if (old + 1 > fp.max_T) capped = 1;
                }
            }
        }
    }
    __syncthreads();
    if (tid == 0) {
        const int status = (act_in > fp.max_T || capped) ? GR_ROW_TRUNC_CAP : GR_ROW_OK;
        fp.tcount[2 * row] = cnt_in; fp.tcount[2 * row + 1] = cnt_out;
        RowInfo out = info;
        out.status = status;
        fp.info[row] = out;
        fp.status[row] = status;
    }
}

// ---- acceptance sweep over supports that do not fit LDS (the first experiment of Sec. 7 runs the top-k size up to
// the whole vocabulary).  Behind full_order_kernel with the grid's largest k: kernel A ranks the support by
// decreasing q (ties by token id) and leaves, by ratio rank, p / sum p, q and the q rank of every token, plus the
// q mass of each top-k support of the grid; kernel B takes the masked prefix sums along the ratio order and
// the minimum of F(m) = P_m - Q_m^n for every cell (Thm 3.1, Sec. 5.1).  Only min F is reported, to 1e-5, so these
// sums are parallel float64 scans like those of the LDS-resident sweep.
__global__ __launch_bounds__(kThreads) void full_sweep_rank_kernel(FullParams fp, FullSweep fs) {
    __shared__ SortLds S;
    __shared__ double red[kWaves];
    const int tid = threadIdx.x, row = blockIdx.x;
    const int V = fp.V;
    const size_t vs = static_cast<size_t>(V) + 2;
    const RowInfo info = fp.info[row];
    if (info.status == GR_ROW_BAD) return;
    const int kk = info.support;
    const float* pr = fp.p + static_cast<size_t>(row) * V;
    const float* qr = fp.q + static_cast<size_t>(row) * V;
    const int* order = fp.order + row * vs;
    unsigned long long* k0 = fp.key0 + row * vs; unsigned long long* k1 = fp.key1 + row * vs;
    int* v0 = fp.val0 + row * vs; int* v1 = fp.val1 + row * vs;
    double* pn = fp.pn + row * vs; double* qn = fp.qn + row * vs;
    int* qrank = fp.blk + row * vs;                              // by ratio rank: the token's rank by decreasing q
    for (int r0 = tid; r0 < kk; r0 += 4 * kThreads) {
        int id[4]; float qv[4], pv[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) { const int r = r0 + j * kThreads; id[j] = r < kk ? order[r] : 0; }
#pragma unroll
        for (int j = 0; j < 4; ++j) { qv[j] = qr[id[j]]; pv[j] = pr[id[j]]; }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int r = r0 + j * kThreads;
            if (r < kk) {
                const unsigned long long qb = static_cast<unsigned long long>(~__float_as_uint(qv[j]) & 0x7FFFFFFFu);
                k0[r] = (qb << 24) | static_cast<unsigned long long>(id[j]);
                v0[r] = r;
                pn[r] = static_cast<double>(pv[j]) / info.p_total;
                qn[r] = static_cast<double>(qv[j]);
            }
        }
    }
    __syncthreads();
    const int res = block_radix_sort(k0, v0, k1, v1, kk, S);
    const int* sorted = res ? v1 : v0;
    // sorted[j] = ratio rank of the token of q rank j; the q mass of the first k of them for every k of the grid
    double part[kSweepMaxK];
#pragma unroll
    for (int a = 0; a < kSweepMaxK; ++a) part[a] = 0.0;
    for (int j = tid; j < kk; j += kThreads) {
        const int r = sorted[j];
        qrank[r] = j;
        const double qv = qn[r];
#pragma unroll
        for (int a = 0; a < kSweepMaxK; ++a) if (a < fs.nk && j < fs.ks[a]) part[a] += qv;
    }
#pragma unroll
    for (int a = 0; a < kSweepMaxK; ++a) {
        const double t = block_sum(part[a], red);
        if (tid == 0 && a < fs.nk) fs.mass[row * kSweepMaxK + a] = t;
    }
}

__global__ __launch_bounds__(kThreads) void full_sweep_scan_kernel(FullParams fp, FullSweep fs) {
    __shared__ double wtot[2][kWaves];
    __shared__ double cell[kSweepMaxK][kSweepMaxN][kWaves];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, row = blockIdx.x;
    const size_t vs = static_cast<size_t>(fp.V) + 2;
    const int cells = fs.nk * fs.nn;
    float* out = fs.accept_prob + static_cast<size_t>(row) * cells;
    const RowInfo info = fp.info[row];
    if (info.status == GR_ROW_BAD) {
        for (int c = tid; c < cells; c += kThreads) out[c] = __uint_as_float(0x7fc00000u);
        if (tid == 0) fs.status[row] = GR_ROW_BAD;
        return;
    }
    const int kk = info.support;
    const double* pn = fp.pn + row * vs; const double* qn = fp.qn + row * vs;
    const int* qrank = fp.blk + row * vs;
    for (int c = tid; c < kSweepMaxK * kSweepMaxN * kWaves; c += kThreads) (&cell[0][0][0])[c] = 0.0;   // F(0) = 0: the empty prefix
    double carryP[kSweepMaxK], carryS[kSweepMaxK], mass[kSweepMaxK];
#pragma unroll
    for (int a = 0; a < kSweepMaxK; ++a) { carryP[a] = 0.0; carryS[a] = 0.0; mass[a] = a < fs.nk ? fs.mass[row * kSweepMaxK + a] : 1.0; }
    __syncthreads();
    for (int t0 = 0; t0 < kk; t0 += 4 * kThreads) {             // 1024 ranks per round, four consecutive ones per thread
        double pv[4], qv[4]; int qrk[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int r = t0 + 4 * tid + j;
            pv[j] = r < kk ? pn[r] : 0.0; qv[j] = r < kk ? qn[r] : 0.0; qrk[j] = r < kk ? qrank[r] : 0x7fffffff;
        }
#pragma unroll
        for (int a = 0; a < kSweepMaxK; ++a) {
            if (a >= fs.nk) continue;                            // uniform over the workgroup
            const int ka = fs.ks[a];
            double lp[4], ls[4];
            double accp = 0.0, accs = 0.0;
#pragma unroll
            for (int j = 0; j < 4; ++j) { const bool on = qrk[j] < ka; accp += on ? pv[j] : 0.0; accs += on ? qv[j] : 0.0; lp[j] = accp; ls[j] = accs; }
            // exclusive prefix of the threads' sums over the workgroup
            double ip = accp, is = accs;
            for (int o = 1; o < 64; o <<= 1) {
                const double up = __shfl_up(ip, o), us = __shfl_up(is, o);
                if (lane >= o) { ip += up; is += us; }
            }
            if (lane == 63) { wtot[0][wv] = ip; wtot[1][wv] = is; }
            __syncthreads();
            double bp = carryP[a] + (ip - accp), bs = carryS[a] + (is - accs), tp = 0.0, ts = 0.0;
#pragma unroll
            for (int w = 0; w < kWaves; ++w) { if (w < wv) { bp += wtot[0][w]; bs += wtot[1][w]; } tp += wtot[0][w]; ts += wtot[1][w]; }
            carryP[a] += tp; carryS[a] += ts;
            const double inv = 1.0 / mass[a];
            for (int b = 0; b < fs.nn; ++b) {
                double m = 0.0;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    // a rank outside this support repeats the prefix before it; ranks beyond the support add nothing
                    const double F = (bp + lp[j]) - ipow((bs + ls[j]) * inv, fs.ns[b]);
                    m = fmin(m, (t0 + 4 * tid + j < kk) ? F : 0.0);
                }
                m = wave_min(m);
                if (lane == 0) cell[a][b][wv] = fmin(cell[a][b][wv], m);
            }
            __syncthreads();                                     // wtot is rewritten by the next k
        }
    }
    __syncthreads();
    for (int c = tid; c < cells; c += kThreads) {
        const int a = c / fs.nn, b = c % fs.nn;
        double t = cell[a][b][0];
        for (int w = 1; w < kWaves; ++w) t = fmin(t, cell[a][b][w]);
        out[c] = static_cast<float>(1.0 + t);
    }
    if (tid == 0) fs.status[row] = GR_ROW_OK;
}

void launch_full_sweep(const FullParams& fp, const FullSweep& fs, hipStream_t stream) {
    hipLaunchKernelGGL(full_order_kernel, dim3(fp.B), dim3(kThreads), 0, stream, fp);
    hipLaunchKernelGGL(full_sweep_rank_kernel, dim3(fp.B), dim3(kThreads), 0, stream, fp, fs);
    hipLaunchKernelGGL(full_sweep_scan_kernel, dim3(fp.B), dim3(kThreads), 0, stream, fp, fs);
}

void launch_full_prologue(const FullParams& fp, hipStream_t stream) {
    hipLaunchKernelGGL(full_order_kernel, dim3(fp.B), dim3(kThreads), 0, stream, fp);
    hipLaunchKernelGGL(full_scan_kernel, dim3(fp.B), dim3(kThreads), 0, stream, fp);
    hipLaunchKernelGGL(full_trunc_kernel, dim3(fp.B), dim3(kThreads), 0, stream, fp);
}

}  // namespace gr
