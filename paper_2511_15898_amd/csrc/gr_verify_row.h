// One row's verification: the transport slice pi(.|drafts) (Eq. "cases", Eq. "approx-c") and the single inverse-CDF
// draw from it.  Shared by verify_kernel and by the solve kernel, which can run it for its own row as soon as the
// row's policy is written.  Exactly kThreads (256) threads of a workgroup call verify_row together.
#pragma once
#include "gr_internal.h"

namespace gr {
namespace {

enum Mode { kOuter = 0, kInner = 1, kFallback = 2, kBadDraft = 3 };

struct Slice {
    int nd;                    // number of distinct drafts
    int tok[GR_MAX_N];         // in order of first appearance
    int pos[GR_MAX_N];         // rank position in the support, -1 if absent
    double pi[GR_MAX_N];       // probability of each distinct draft
    double wv[GR_MAX_N];       // its weight, its probability under p, its block (loaded by one thread each)
    double pv[GR_MAX_N];
    int bv[GR_MAX_N];
    double acc;                // sum of pi over the drafts
    double scale;              // multiplies the residual weight of every other token
    int mode;
};

// Entry t of the row that `info` describes, before the division by info.p_total: the stored probability, or, for a
// row given as logits (App. A: temperature only changes how p comes from the logits), exp((t - p_ref) / T).
__device__ __forceinline__ double p_entry(const float* prow, int t, const RowInfo& info) {
    const double x = static_cast<double>(prow[t]);
    return info.inv_temp > 0.0 ? exp((x - info.p_ref) * info.inv_temp) : x;
}

// All threads call; result in LDS `S`.  order/block/weight: this row's policy arrays.
// rank_of: token -> rank of a full-vocabulary policy (nullptr for a top-k policy, whose ranks are
// found by a scan of `order`).
__device__ void build_slice(Slice& S, const RowInfo& info, const int* order, const int* block,
                            const double* weight, const int* rank_of, const int* drafts, int n,
                            const float* prow, int V) {
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
    if (info.status == GR_ROW_OK) {
        if (rank_of) {
            if (tid < S.nd) S.pos[tid] = rank_of[S.tok[tid]];
        } else if (tid < kk) {
            const int t = order[tid];
            for (int i = 0; i < S.nd; ++i) if (S.tok[i] == t) S.pos[i] = tid;
        }
    }
    __syncthreads();
    if (tid < S.nd) {
        const int pos = S.pos[tid];
        S.wv[tid] = pos >= 0 ? weight[pos] : 0.0;
        S.bv[tid] = pos >= 0 ? block[pos] : -1;
        S.pv[tid] = p_entry(prow, S.tok[tid], info);
    }
    __syncthreads();
    if (tid == 0) {
        const int nd = S.nd;
        if (S.mode == kBadDraft) {
            for (int i = 0; i < nd; ++i) S.pi[i] = 0.0;
            S.acc = 0.0; S.scale = 0.0;
        } else if (info.status != GR_ROW_OK) {
            double a = 0.0;
            for (int i = 0; i < nd; ++i) { S.pi[i] = S.pv[i] / info.p_total; a += S.pi[i]; }
            S.acc = a; S.scale = 1.0; S.mode = kFallback;
        } else {
            int mmax = -1; bool missing = false;
            for (int i = 0; i < nd; ++i) { missing |= S.pos[i] < 0; mmax = max(mmax, S.pos[i]); }
            if (missing) {
                for (int i = 0; i < nd; ++i) S.pi[i] = 0.0;
                S.acc = 0.0; S.scale = 0.0; S.mode = kBadDraft;
            } else if (mmax < info.h) {
                double s = 0.0;
                for (int i = 0; i < nd; ++i) s += S.wv[i];
                const double den = 1.0 + s;
                for (int i = 0; i < nd; ++i) S.pi[i] = S.wv[i] / den;
                S.acc = 1.0 - 1.0 / den;
                S.scale = info.res_total > 0.0 ? (1.0 / den) / info.res_total : 0.0;
                S.mode = kInner;
            } else {
                int b = -1;
                for (int i = 0; i < nd; ++i) if (S.pos[i] == mmax) b = S.bv[i];
                double s = 0.0; int members = 0;
                for (int i = 0; i < nd; ++i)
                    if (S.pos[i] >= info.h && S.bv[i] == b) { s += S.wv[i]; ++members; }
                for (int i = 0; i < nd; ++i) {
                    const bool in = S.pos[i] >= info.h && S.bv[i] == b;
                    S.pi[i] = in ? (s > 0.0 ? S.wv[i] / s : 1.0 / members) : 0.0;
                }
                S.acc = 1.0; S.scale = 0.0; S.mode = kOuter;
            }
        }
    }
    __syncthreads();
}

// Four consecutive probabilities from token t0 on; entries at or beyond `end` read as zero.
__device__ __forceinline__ float4 load4(const float* prow, int t0, int end, bool vec) {
    if (vec && t0 + 3 < end) return *reinterpret_cast<const float4*>(prow + t0);
    float4 r = make_float4(0.f, 0.f, 0.f, 0.f);
    if (t0 < end) r.x = prow[t0];
    if (t0 + 1 < end) r.y = prow[t0 + 1];
    if (t0 + 2 < end) r.z = prow[t0 + 2];
    if (t0 + 3 < end) r.w = prow[t0 + 3];
    return r;
}


// This row's policy arrays (already offset to the row) and the piece sums of p that came with the select pass.
struct RowPolicy {
    const int* o; const int* bl; const double* wt; const double* rh;   // order, block, weight, rho by rank
    const int* rk; const double* rid;                                 // full-vocabulary policies: rank and residual by token id
    const double* pieces; const float* prefs;                         // sums of p over pieces of 256 tokens (or nullptr), their references
};

// LDS of verify_row.
struct VerifyLds {
    Slice S;
    double w[256];
    double red[kWaves];
    double wtot[kWaves];
    double seg[64];
    int chosen;
};

// prow: the row of p (V entries); drafts: its n drafts; token/accepted: where the row's result goes.
__device__ inline void verify_row(VerifyLds& vl, const float* prow, int V, int n, const RowPolicy& rp, const RowInfo& info,
                                  const int* drafts, float uniform, int* token, unsigned char* accepted) {
    Slice& S = vl.S;
    double* const w = vl.w; double* const red = vl.red; double* const wtot = vl.wtot; double* const seg = vl.seg;
    int& chosen = vl.chosen;
    const int tid = threadIdx.x;
    const int* o = rp.o; const int* bl = rp.bl; const double* wt = rp.wt; const double* rh = rp.rh;
    const int* rk = rp.rk; const double* rid = rp.rid;
    if (info.status == GR_ROW_BAD) {
        if (tid == 0) { *token = -1; *accepted = 0; }
        return;
    }
    build_slice(S, info, o, bl, wt, rk, drafts, n, prow, V);
    const double u = static_cast<double>(uniform);
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
        if (tid == 0) { *token = -1; *accepted = 0; }
        return;
    }
    if (first >= 0) {
        if (tid == 0) { *token = first; *accepted = 1; }
        return;
    }
    // ---- not among the drafts: the remaining tokens by ascending id.  The range that holds the draw
    // is narrowed level by level: it is cut into at most 64 pieces, every wave sums whole pieces with
    // coalesced loads (no barrier inside), a scan over the piece sums picks the piece, and the last
    // 256 tokens are scanned one per thread.  The p row is read once plus two short re-reads.
    const int lane = tid & 63, wvv = tid >> 6;
    const double f = S.scale / info.p_total;
    const bool vec = (reinterpret_cast<uintptr_t>(prow) & 15) == 0;
    // weight of a token that is not f * p: the support (residual rho outside H*, none inside) when
    // the drafts all lie in H*; the drafts themselves (listed first) in the fallback
    // a full-vocabulary policy whose drafts all lie in H* spreads the slack over scale * rho_id[t]
    const bool dense = rid != nullptr && S.mode == kInner;
    const double* pieces = dense ? nullptr : rp.pieces;
    const bool from_logits = info.inv_temp > 0.0;           // piece sums are then relative to a reference of their own
    const float* prefs = (pieces && from_logits) ? rp.prefs : nullptr;
    const int n_special = dense ? 0 : (S.mode == kInner ? info.support : S.nd);
    int sp_tok = -1; double sp_w = 0.0;
    if (tid < n_special) {
        if (S.mode == kInner) { sp_tok = o[tid]; sp_w = tid >= info.h ? S.scale * rh[tid] : 0.0; }
        else { sp_tok = S.tok[tid]; sp_w = 0.0; }
    }
    const double sp_delta = sp_tok >= 0 ? sp_w - f * p_entry(prow, sp_tok, info) : 0.0;
    int lo = 0, len = V;
    double cum = c;
    bool beyond = false;                      // the draw lies beyond the total by rounding: take the last token with mass
    while (len > 256) {
        const int g = (len + 256 * 64 - 1) / (256 * 64);
        const int cs = 256 * g;
        const int np = (len + cs - 1) / cs;
        const int end = lo + len;
        if (pieces) {
            // the sums of p over every 256 tokens came with the select pass: no read of the row here
            const int npv = (V + 255) >> 8;
            for (int pc = wvv; pc < np; pc += kWaves) {
                double sa = 0.0;
                for (int sub = lane; sub < g; sub += 64) {
                    const int idx = (lo >> 8) + pc * g + sub;
                    if (idx < npv) sa += prefs ? pieces[idx] * exp((static_cast<double>(prefs[idx]) - info.p_ref) * info.inv_temp) : pieces[idx];
                }
                sa = wave_sum(sa);
                if (lane == 0) seg[pc] = f * sa;
            }
        } else if (dense) {
            for (int pc = wvv; pc < np; pc += kWaves) {
                double sa = 0.0;
#pragma unroll 4
                for (int sub = 0; sub < g; ++sub) {
                    const int t0 = lo + pc * cs + sub * 256 + lane * 4;
#pragma unroll
                    for (int j = 0; j < 4; ++j) if (t0 + j < end) sa += rid[t0 + j];
                }
                sa = wave_sum(sa);
                if (lane == 0) seg[pc] = S.scale * sa;
            }
        } else if (from_logits) {                       // no piece sums on this handle: exponentials of the whole range
            for (int pc = wvv; pc < np; pc += kWaves) {
                double sa = 0.0;
                for (int sub = 0; sub < g; ++sub) {
                    const int t0 = lo + pc * cs + sub * 256 + lane * 4;
#pragma unroll
                    for (int j = 0; j < 4; ++j) if (t0 + j < end) sa += p_entry(prow, t0 + j, info);
                }
                sa = wave_sum(sa);
                if (lane == 0) seg[pc] = f * sa;
            }
        } else
        // two pieces per round and up to eight loads of each in flight: one workgroup streams the row,
        // so the walk is bound by load latency, not by bandwidth
        for (int pc = wvv; pc < np; pc += 2 * kWaves) {
            double sa = 0.0, sb = 0.0;
            const int pb = pc + kWaves;
            for (int sub0 = 0; sub0 < g; sub0 += 8) {
                float4 va[8], vb[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int ta = lo + pc * cs + (sub0 + j) * 256 + lane * 4;
                    va[j] = sub0 + j < g ? load4(prow, ta, end, vec) : make_float4(0.f, 0.f, 0.f, 0.f);
                }
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int tb = lo + pb * cs + (sub0 + j) * 256 + lane * 4;
                    vb[j] = (pb < np && sub0 + j < g) ? load4(prow, tb, end, vec) : make_float4(0.f, 0.f, 0.f, 0.f);
                }
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    sa += (static_cast<double>(va[j].x) + static_cast<double>(va[j].y)) + (static_cast<double>(va[j].z) + static_cast<double>(va[j].w));
                    sb += (static_cast<double>(vb[j].x) + static_cast<double>(vb[j].y)) + (static_cast<double>(vb[j].z) + static_cast<double>(vb[j].w));
                }
            }
            sa = wave_sum(sa); sb = wave_sum(sb);
            if (lane == 0) { seg[pc] = f * sa; if (pb < np) seg[pb] = f * sb; }
        }
        __syncthreads();
        if (sp_tok >= lo && sp_tok < end) atomicAdd(&seg[(sp_tok - lo) / cs], sp_delta);
        __syncthreads();
        if (wvv == 0) {
            const double v = lane < np ? fmax(seg[lane], 0.0) : 0.0;
            double incl = v;
            for (int off = 1; off < 64; off <<= 1) { const double up = __shfl_up(incl, off); if (lane >= off) incl += up; }
            const bool pos = v > 0.0;
            const unsigned long long hits = __ballot(pos && !beyond && u < cum + incl);
            const unsigned long long poss = __ballot(pos);
            int pick = -1, past = 0;
            if (hits) pick = __ffsll(static_cast<long long>(hits)) - 1;
            else if (poss) { pick = 63 - __clzll(static_cast<long long>(poss)); past = 1; }
            if (lane == (pick < 0 ? 0 : pick)) { chosen = pick; red[0] = cum + (incl - v); wtot[0] = past; }
        }
        __syncthreads();
        const int pick = chosen;
        if (pick < 0) break;
        cum = red[0];
        beyond = beyond || wtot[0] != 0.0;
        lo += pick * cs;
        len = min(cs, end - lo);
        __syncthreads();
    }
    if (len > 256) {                          // no residual mass at all: keep the last draft with mass
        if (tid == 0) {
            int t = -1;
            for (int i = 0; i < S.nd; ++i) if (S.pi[i] > 0.0) t = S.tok[i];
            *token = t; *accepted = t >= 0 ? 1 : 0;
        }
        return;
    }
    {
        const int t = lo + tid;
        w[tid] = tid < len ? (dense ? S.scale * rid[t] : f * p_entry(prow, t, info)) : 0.0;
        __syncthreads();
        if (sp_tok >= lo && sp_tok < lo + len) w[sp_tok - lo] = sp_w;
        __syncthreads();
        const double mw = fmax(w[tid], 0.0);
        double incl = mw;
        for (int off = 1; off < 64; off <<= 1) { const double up = __shfl_up(incl, off); if (lane >= off) incl += up; }
        if (lane == 63) wtot[wvv] = incl;
        __syncthreads();
        double bef = 0.0;
        for (int w2 = 0; w2 < wvv; ++w2) bef += wtot[w2];
        const bool pos = mw > 0.0;
        const bool hitme = pos && !beyond && u < cum + bef + incl;
        const int hm = static_cast<int>(block_min(hitme ? static_cast<double>(t) : 2147483647.0, red));
        const int lm = static_cast<int>(block_max(pos ? static_cast<double>(t) : -1.0, red));
        if (tid == 0) {
            int t_out = hm != 0x7fffffff ? hm : lm;
            bool acc = false;
            if (t_out < 0) {                  // V <= 256 and no residual mass
                for (int i = 0; i < S.nd; ++i) if (S.pi[i] > 0.0) t_out = S.tok[i];
                acc = t_out >= 0;
            }
            *token = t_out; *accepted = acc ? 1 : 0;
        }
    }
}

}  // namespace
}  // namespace gr
