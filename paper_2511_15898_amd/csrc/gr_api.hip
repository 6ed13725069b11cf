// C ABI of the Global Resolution verifier: handle, argument checks, kernel launches.
#include <new>
#include <vector>

#include "gr_internal.h"

using namespace gr;

namespace { constexpr int kProfSlots = 512; }

struct gr_handle_s {
    int max_B = 0, max_V = 0;
    int k_cap = 0;                 // largest support (top-k, or max_V for whole rows) the handle was created for
    int max_n = GR_MAX_N;
    int max_iter = 1000, max_T = GR_MAX_T;
    double rel_tol = 1e-8;
    double tail_mass = 0.0;        // nucleus cut of the draft on the HBM-resident path
    int device = 0;
    // scratch of the select kernel
    unsigned long long* cand = nullptr; int* cand_count = nullptr;
    double* part_psum = nullptr; double* part_qsum = nullptr; int* part_bad = nullptr;
    double* newton_ws = nullptr;   // [max_B, kMaxT * (kMaxT + 1)] Jacobian scratch of the solver's Newton fallback
    double* piece_psum = nullptr; int piece_stride = 0;   // float64 sums of p per 256 tokens, [max_B, piece_stride]
    float* piece_pref = nullptr; float* part_pref = nullptr;   // rows given as logits: the references of the piece sums and of the slices' sums
    // policy object of the last solve
    int* order = nullptr; int* block = nullptr; double* weight = nullptr; double* rho = nullptr; double* pnorm = nullptr;
    RowInfo* info = nullptr;
    // optional per-kernel timing (gr_config.flags bit 0): events around every launch, read back
    // by gr_profile_read
    bool profile = false;
    int prof_stride = 1, prof_tick = 0;   // events are recorded on every prof_stride-th solve (and the verify that follows it)
    bool prof_now = false;
    hipEvent_t ev[kProfSlots][5] = {};
    int prof_count = 0;
    // full-vocabulary path: workspace (allocated by gr_create when k_cap exceeds GR_MAX_SUPPORT) and the arguments of the last such solve
    void* full_ws = nullptr; size_t full_ws_bytes = 0;
    double* sweep_mass = nullptr;  // [max_B, kSweepMaxK] q mass of each top-k support of a sweep that runs in the workspace
    FullParams full = {};
    bool full_mode = false;
    // staging of gr_tree_walk (allocated by its first call): gathered rows, drafts, uniforms, results, row offsets
    float* tw_p = nullptr; float* tw_q = nullptr; int* tw_drafts = nullptr; float* tw_u = nullptr; float* tw_temp = nullptr; int* tw_tok = nullptr;
    unsigned char* tw_ok = nullptr; long long* tw_idx = nullptr; float* tw_acc = nullptr; int* tw_status = nullptr;
    // last solve
    bool solved = false;
    const float* p = nullptr;
    int B = 0, V = 0, n = 0;
};

namespace {

void mark(gr_handle h, int which, hipStream_t stream) {
    if (which == 0) h->prof_now = h->profile && (h->prof_tick++ % h->prof_stride == 0);
    if (h->prof_now && h->prof_count < kProfSlots) (void)hipEventRecord(h->ev[h->prof_count][which], stream);
}

template <typename T>
bool dev_alloc(T** ptr, size_t count) {
    return hipMalloc(reinterpret_cast<void**>(ptr), count * sizeof(T)) == hipSuccess;
}

void free_all(gr_handle h) {
    void* ptrs[] = {h->cand, h->cand_count, h->part_psum, h->part_qsum, h->part_bad, h->piece_psum, h->piece_pref, h->part_pref, h->tw_p, h->tw_q, h->tw_drafts, h->tw_u, h->tw_temp, h->tw_tok, h->tw_ok, h->tw_idx, h->tw_acc, h->tw_status, h->sweep_mass, h->newton_ws, h->order, h->block,
                    h->weight, h->rho, h->pnorm, h->info};
    for (void* ptr : ptrs) (void)hipFree(ptr);
    (void)hipFree(h->full_ws);
    if (h->profile)
        for (auto& slot : h->ev)
            for (auto& e : slot)
                if (e) (void)hipEventDestroy(e);
}

// Number of workgroups that share a row in the select kernel: enough groups to keep every CU's
// memory pipeline busy (about 8 per CU), slices no shorter than 4 tiles.
int choose_splits(int B, int V) {
    int s = 2048 / (B > 0 ? B : 1);
    if (s < 1) s = 1;
    if (s > kMaxSplits) s = kMaxSplits;
    while (s > 1 && V / s < 4 * kSelTile) --s;
    return s;
}

PolicyView policy_view(gr_handle h) {
    PolicyView pv;
    if (h->full_mode) {
        const FullParams& f = h->full;
        pv.order = f.order; pv.block = f.blk; pv.weight = f.weight; pv.rho = f.rho;
        pv.rank_of = f.rank_of; pv.rho_id = f.rho_id; pv.stride = static_cast<size_t>(h->V) + 2;
        pv.piece_psum = nullptr; pv.piece_stride = 0; pv.piece_pref = nullptr;
    } else {
        pv.order = h->order; pv.block = h->block; pv.weight = h->weight; pv.rho = h->rho;
        pv.rank_of = nullptr; pv.rho_id = nullptr; pv.stride = kMaxSupport;
        pv.piece_psum = h->piece_psum; pv.piece_stride = h->piece_stride; pv.piece_pref = h->piece_pref;
    }
    return pv;
}

constexpr size_t kFullPad = 256;
size_t full_ws_bytes(size_t rows, size_t vs) { return rows * vs * kFullBytesPerToken + 40 * kFullPad + rows * 3 * sizeof(int); }

// Carve the workspace of the full-vocabulary path (allocated once by gr_create) for a batch of B rows of V tokens.
int prepare_full(gr_handle h, int B, int V) {
    const size_t vs = static_cast<size_t>(V) + 2, rows = static_cast<size_t>(B);
    const size_t per_array_pad = kFullPad;
    if (full_ws_bytes(rows, vs) > h->full_ws_bytes) return GR_EINVAL;      // cannot happen for B <= max_B, V <= max_V
    unsigned char* cur = static_cast<unsigned char*>(h->full_ws);
    auto take = [&](size_t bytes) { void* r = cur; cur += (bytes + per_array_pad - 1) / per_array_pad * per_array_pad; return r; };
    FullParams& f = h->full;
    const size_t cnt = rows * vs;
    f.key0 = static_cast<unsigned long long*>(take(cnt * 8)); f.key1 = static_cast<unsigned long long*>(take(cnt * 8));
    f.val0 = static_cast<int*>(take(cnt * 4)); f.val1 = static_cast<int*>(take(cnt * 4));
    f.order = static_cast<int*>(take(cnt * 4)); f.byq = static_cast<int*>(take(cnt * 4));
    double** dbl[] = {&f.pn, &f.qn, &f.P, &f.Q, &f.F, &f.rho, &f.tgt, &f.weight, &f.rho_id};
    for (double** d : dbl) *d = static_cast<double*>(take(cnt * 8));
    int** ints[] = {&f.flag, &f.blk, &f.blo, &f.inT, &f.bcount, &f.rank_of};
    for (int** d : ints) *d = static_cast<int*>(take(cnt * 4));
    f.nblk = static_cast<int*>(take(rows * 4)); f.tcount = static_cast<int*>(take(rows * 8));
    return GR_OK;
}

}  // namespace

// ---- allocation-free sweep: the selection scratch lives in the device image.
namespace {

constexpr size_t kNoAllocRows = GR_NOALLOC_MAX_B;
constexpr size_t kNaCand = 0;                                                                  // u64 [rows, kMaxSplits, kMaxSupport]
constexpr size_t kNaPsum = kNaCand + kNoAllocRows * kMaxSplits * kMaxSupport * sizeof(unsigned long long);   // f64 [rows, kMaxSplits]
constexpr size_t kNaQsum = kNaPsum + kNoAllocRows * kMaxSplits * sizeof(double);              // f64 [rows, kMaxSplits]
constexpr size_t kNaCount = kNaQsum + kNoAllocRows * kMaxSplits * sizeof(double);             // i32 [rows, kMaxSplits]
constexpr size_t kNaBad = kNaCount + kNoAllocRows * kMaxSplits * sizeof(int);                 // i32 [rows, kMaxSplits]
constexpr size_t kNaBytes = kNaBad + kNoAllocRows * kMaxSplits * sizeof(int);

static __device__ __align__(256) unsigned char scratch[kNaBytes];

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};       // device address of `scratch` on each GPU, looked up once per device

// The address of this device's copy of `scratch` (host code must never pass the array's name to a kernel).
int scratch_address(unsigned char** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return GR_EHIP;
    void* ptr = __atomic_load_n(&g_scratch_ptr[dev], __ATOMIC_ACQUIRE);
    if (!ptr) {
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) { (void)hipGetLastError(); return GR_EHIP; }
        __atomic_store_n(&g_scratch_ptr[dev], ptr, __ATOMIC_RELEASE);      // every thread finds the same address
    }
    *out = static_cast<unsigned char*>(ptr);
    return GR_OK;
}

// Argument checks and grid of a sweep, shared by both entry points.
int fill_sweep(SweepParams& sw, const int* ks, int nk, const int* ns, int nn, int V) {
    if (nk < 1 || nk > kSweepMaxK || nn < 1 || nn > kSweepMaxN) return GR_EINVAL;
    sw.kmax = 0;
    for (int i = 0; i < nk; ++i) {
        if (ks[i] < 1 || ks[i] > kMaxSupport) return GR_EINVAL;
        sw.ks[i] = ks[i];
        if (ks[i] > sw.kmax) sw.kmax = ks[i];
    }
    for (int i = 0; i < nn; ++i) {
        if (ns[i] < 1 || ns[i] > kSweepMaxDrafts) return GR_EINVAL;
        sw.ns[i] = ns[i];
    }
    if (sw.kmax > V) sw.kmax = V;                        // a top-k of V or more keeps every positive entry
    for (int i = nk; i < kSweepMaxK; ++i) sw.ks[i] = 0;
    for (int i = nn; i < kSweepMaxN; ++i) sw.ns[i] = 1;
    sw.nk = nk; sw.nn = nn; sw.V = V;
    return GR_OK;
}

// The HBM-resident path (a support above GR_MAX_SUPPORT: no top-k, or a large one) of gr_solve (temperature == nullptr)
// and of gr_solve_logits.
int solve_in_hbm(gr_handle h, const float* p, const float* q, const float* temperature, const float* draft_temperature, int n, int k_eff, float tol, int B, int V,
                 float* accept_prob, int* status, hipStream_t stream) {
    if (V >= (1 << 24)) return GR_EUNSUPPORTED;
    h->solved = false;
    const int rc = prepare_full(h, B, V);
    if (rc != GR_OK) return rc;
    FullParams& f = h->full;
    f.p = p; f.q = q; f.B = B; f.V = V; f.n = n; f.k = k_eff; f.max_T = h->max_T; f.max_iter = h->max_iter;
    f.tau = static_cast<double>(tol); f.rel_tol = h->rel_tol; f.tail_mass = h->tail_mass;
    f.logits = temperature ? 1 : 0; f.temperature = temperature; f.draft_temperature = draft_temperature;
    f.info = h->info; f.accept_prob = accept_prob; f.status = status; f.newton_ws = h->newton_ws;
    mark(h, 0, stream);
    launch_full_prologue(f, stream);
    if (hipGetLastError() != hipSuccess) return GR_EHIP;
    mark(h, 1, stream);
    if (launch_full_programs(f, stream) != hipSuccess) return GR_EHIP;
    mark(h, 2, stream);
    h->solved = true; h->full_mode = true; h->p = p; h->B = B; h->V = V; h->n = n;
    return GR_OK;
}

// The LDS-resident path of gr_solve (temperature == nullptr: p and q are probabilities) and of gr_solve_logits.
// With drafts (and uniforms, token, accepted) the solve kernel also verifies every row; otherwise all four are nullptr.
int solve_in_lds(gr_handle h, const float* p, const float* q, const float* temperature, const float* draft_temperature, int n, int k_eff, float tol, int B, int V,
                 float* accept_prob, int* status, hipStream_t stream, const int* drafts = nullptr, const float* uniforms = nullptr,
                 int* token = nullptr, unsigned char* accepted = nullptr) {
    h->full_mode = false;
    const int splits = choose_splits(B, V);
    int slice_len = (V + splits - 1) / splits;
    slice_len = (slice_len + kSelTile - 1) / kSelTile * kSelTile;
    h->solved = false;
    mark(h, 0, stream);
    if (temperature)
        launch_select_logits(p, q, temperature, B, V, k_eff, splits, slice_len, h->cand, h->cand_count, h->part_psum, h->part_qsum,
                             h->part_bad, h->part_pref, h->piece_psum, h->piece_pref, h->piece_stride, stream);
    else
        launch_select(p, q, B, V, k_eff, splits, slice_len, h->cand, h->cand_count, h->part_psum, h->part_qsum,
                      h->part_bad, h->piece_psum, h->piece_stride, stream);
    if (hipGetLastError() != hipSuccess) return GR_EHIP;
    mark(h, 1, stream);
    SolveParams sp;
    sp.p = p; sp.q = q; sp.B = B; sp.V = V; sp.n = n; sp.k = k_eff; sp.splits = splits;
    sp.tau = static_cast<double>(tol); sp.rel_tol = h->rel_tol; sp.max_iter = h->max_iter; sp.max_T = h->max_T;
    sp.tail_mass = temperature ? 0.0 : h->tail_mass;
    sp.cand = h->cand; sp.cand_count = h->cand_count; sp.part_psum = h->part_psum; sp.part_qsum = h->part_qsum;
    sp.part_bad = h->part_bad;
    sp.logits = temperature ? 1 : 0; sp.temperature = temperature; sp.part_pref = h->part_pref; sp.draft_temperature = draft_temperature;
    sp.order = h->order; sp.block = h->block; sp.weight = h->weight; sp.rho = h->rho; sp.pnorm = h->pnorm;
    sp.info = h->info; sp.accept_prob = accept_prob; sp.status = status; sp.newton_ws = h->newton_ws;
    sp.v_drafts = drafts; sp.v_uniforms = uniforms; sp.v_token = token; sp.v_accepted = accepted;
    sp.piece_psum = h->piece_psum; sp.piece_stride = h->piece_stride; sp.piece_pref = h->piece_pref;
    if (launch_solve(sp, stream) != hipSuccess) return GR_EHIP;
    mark(h, 2, stream);
    h->solved = true; h->p = p; h->B = B; h->V = V; h->n = n;
    return GR_OK;
}

}  // namespace

extern "C" int gr_create(gr_handle* out, int max_B, int max_V, int max_k, int max_n, const gr_config* cfg) {
    if (!out || max_B <= 0 || max_V <= 0) return GR_EINVAL;
    if (max_n < 1 || max_n > GR_MAX_N) return GR_EINVAL;
    const int k_cap = (max_k <= 0 || max_k >= max_V) ? max_V : max_k;
    if (k_cap > kMaxSupport && max_V >= (1 << 24)) return GR_EUNSUPPORTED;
    if (cfg && (cfg->flags & ~GR_FLAG_PROFILE) != 0) return GR_EINVAL;
    gr_handle h = new (std::nothrow) gr_handle_s();
    if (!h) return GR_ENOMEM;
    h->max_B = max_B; h->max_V = max_V; h->k_cap = k_cap; h->max_n = max_n;
    if (cfg) {
        if (cfg->max_iter > 0) h->max_iter = cfg->max_iter;
        if (cfg->max_T > 0 && cfg->max_T <= GR_MAX_T) h->max_T = cfg->max_T;
        if (cfg->rel_tol > 0.0) h->rel_tol = cfg->rel_tol;
        if (!(cfg->tail_mass >= 0.0) || !(cfg->tail_mass < 1.0)) { delete h; return GR_EINVAL; }
        h->tail_mass = cfg->tail_mass;
    }
    if (hipGetDevice(&h->device) != hipSuccess) { delete h; return GR_EHIP; }
    if (solve_kernel_setup() != hipSuccess) { delete h; return GR_EHIP; }
    { unsigned char* na = nullptr; (void)scratch_address(&na); }      // so that gr_accept_sweep_noalloc finds its array later
    const size_t rows = static_cast<size_t>(max_B);
    bool ok = dev_alloc(&h->cand, rows * kMaxSplits * kMaxSupport) && dev_alloc(&h->cand_count, rows * kMaxSplits) &&
              dev_alloc(&h->part_psum, rows * kMaxSplits) && dev_alloc(&h->part_qsum, rows * kMaxSplits) &&
              dev_alloc(&h->part_bad, rows * kMaxSplits) && dev_alloc(&h->order, rows * kMaxSupport) &&
              dev_alloc(&h->block, rows * kMaxSupport) && dev_alloc(&h->weight, rows * kMaxSupport) &&
              dev_alloc(&h->rho, rows * kMaxSupport) && dev_alloc(&h->pnorm, rows * kMaxSupport) &&
              dev_alloc(&h->info, rows);
    h->piece_stride = (max_V + kSelTile - 1) / kSelTile * (kSelTile / 256) + kMaxSplits * (kSelTile / 256);
    ok = ok && dev_alloc(&h->piece_psum, rows * h->piece_stride) && dev_alloc(&h->piece_pref, rows * h->piece_stride) &&
         dev_alloc(&h->part_pref, rows * kMaxSplits);
    ok = ok && dev_alloc(&h->newton_ws, rows * kMaxT * (kMaxT + 1));
    if (ok && k_cap > kMaxSupport) {
        // supports above GR_MAX_SUPPORT live in HBM: 128 bytes per token of max_V and row, held until gr_destroy
        const size_t need = full_ws_bytes(rows, static_cast<size_t>(max_V) + 2);
        ok = hipMalloc(&h->full_ws, need) == hipSuccess && dev_alloc(&h->sweep_mass, rows * kSweepMaxK);
        if (ok) h->full_ws_bytes = need;
    }
    if (!ok) { free_all(h); delete h; (void)hipGetLastError(); return GR_ENOMEM; }
    if (cfg && (cfg->flags & GR_FLAG_PROFILE)) {
        h->profile = true;
        for (auto& slot : h->ev)
            for (auto& e : slot)
                if (hipEventCreate(&e) != hipSuccess) { free_all(h); delete h; return GR_EHIP; }
    }
    *out = h;
    return GR_OK;
}

extern "C" int gr_destroy(gr_handle h) {
    if (!h) return GR_EINVAL;
    free_all(h);
    delete h;
    return GR_OK;
}

namespace {

// The four solve entry points: rows as probabilities (temperature == nullptr) or logits, with or without the rows'
// verification (drafts == nullptr: without).  A support of at most kMaxSupport tokens runs select + solve, the solve
// launch verifying its rows when asked to; a larger one the HBM-resident kernels, then the verify kernel.
int solve_entry(gr_handle h, const float* p, const float* q, const float* temperature, const float* draft_temperature, int n, int k,
                float tol, int B, int V, const int* drafts, const float* uniforms, float* accept_prob, int* status, int* token,
                unsigned char* accepted, void* hip_stream) {
    if (B <= 0 || V <= 0 || B > h->max_B || V > h->max_V) return GR_EINVAL;
    if (n < 1 || n > h->max_n) return GR_EINVAL;
    if (!(tol >= 0.f) || !(tol < 1.f)) return GR_EINVAL;
    const int k_eff = (k <= 0 || k >= V) ? V : k;
    if (temperature && h->tail_mass > 0.0) return GR_EUNSUPPORTED;          // the nucleus cut is defined on probabilities
    if (k_eff > kMaxSupport && k_eff > h->k_cap) return GR_EINVAL;          // the handle holds no workspace for such a support
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (k_eff > kMaxSupport) {
        const int rc = solve_in_hbm(h, p, q, temperature, draft_temperature, n, k_eff, tol, B, V, accept_prob, status, stream);
        return (rc != GR_OK || !drafts) ? rc : gr_verify(h, drafts, uniforms, token, accepted, hip_stream);
    }
    const int rc = solve_in_lds(h, p, q, temperature, draft_temperature, n, k_eff, tol, B, V, accept_prob, status, stream, drafts, uniforms,
                                token, accepted);
    if (rc != GR_OK || !drafts) return rc;
    mark(h, 3, stream);                              // no verify launch of its own: an empty interval in the profile
    mark(h, 4, stream);
    if (h->prof_now && h->prof_count < kProfSlots) ++h->prof_count;
    h->prof_now = false;
    return GR_OK;
}

}  // namespace

extern "C" int gr_solve(gr_handle h, const float* p, const float* q, int n, int k, float tol,
                        int B, int V, float* accept_prob, int* status, void* hip_stream) {
    if (!h || !p || !q || !accept_prob || !status) return GR_EINVAL;
    return solve_entry(h, p, q, nullptr, nullptr, n, k, tol, B, V, nullptr, nullptr, accept_prob, status, nullptr, nullptr, hip_stream);
}

/* gr_solve and gr_verify in one call: see gr_verify.h. */
extern "C" int gr_solve_verify(gr_handle h, const float* p, const float* q, int n, int k, float tol, int B, int V,
                               const int* drafts, const float* uniforms, float* accept_prob, int* status, int* token,
                               unsigned char* accepted, void* hip_stream) {
    if (!h || !p || !q || !accept_prob || !status || !drafts || !uniforms || !token || !accepted) return GR_EINVAL;
    return solve_entry(h, p, q, nullptr, nullptr, n, k, tol, B, V, drafts, uniforms, accept_prob, status, token, accepted, hip_stream);
}

/* Rows given as logits: see gr_verify.h. */
extern "C" int gr_solve_logits(gr_handle h, const float* target_logits, const float* draft_logits, const float* temperature,
                               const float* draft_temperature, int n, int k, float tol, int B, int V, float* accept_prob,
                               int* status, void* hip_stream) {
    if (!h || !target_logits || !draft_logits || !temperature || !accept_prob || !status) return GR_EINVAL;
    return solve_entry(h, target_logits, draft_logits, temperature, draft_temperature, n, k, tol, B, V, nullptr, nullptr, accept_prob, status,
                       nullptr, nullptr, hip_stream);
}

/* gr_solve_logits and gr_verify in one call: see gr_verify.h. */
extern "C" int gr_solve_logits_verify(gr_handle h, const float* target_logits, const float* draft_logits, const float* temperature,
                                      const float* draft_temperature, int n, int k, float tol, int B, int V, const int* drafts,
                                      const float* uniforms, float* accept_prob, int* status, int* token, unsigned char* accepted,
                                      void* hip_stream) {
    if (!h || !target_logits || !draft_logits || !temperature || !accept_prob || !status || !drafts || !uniforms || !token || !accepted)
        return GR_EINVAL;
    return solve_entry(h, target_logits, draft_logits, temperature, draft_temperature, n, k, tol, B, V, drafts, uniforms, accept_prob, status,
                       token, accepted, hip_stream);
}

extern "C" int gr_accept_sweep(gr_handle h, const float* p, const float* q, const int* ks, int nk, const int* ns, int nn,
                               int B, int V, float* accept_prob, int* status, void* hip_stream) {
    if (!h || !p || !q || !ks || !ns || !accept_prob || !status) return GR_EINVAL;
    if (B <= 0 || V <= 0 || B > h->max_B || V > h->max_V) return GR_EINVAL;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    {
        // a top-k above GR_MAX_SUPPORT anywhere in the grid (k <= 0 or k >= V: no top-k): the whole grid runs on
        // the HBM-resident ordering
        int kmax = 0;
        if (nk < 1 || nk > kSweepMaxK || nn < 1 || nn > kSweepMaxN) return GR_EINVAL;
        for (int i = 0; i < nk; ++i) { const int ke = (ks[i] <= 0 || ks[i] >= V) ? V : ks[i]; if (ke > kmax) kmax = ke; }
        if (kmax > kMaxSupport) {
            if (kmax > h->k_cap) return GR_EINVAL;                   // the handle holds no workspace for such a support
            if (V >= (1 << 24)) return GR_EUNSUPPORTED;
            FullSweep fs;
            fs.nk = nk; fs.nn = nn;
            for (int i = 0; i < kSweepMaxK; ++i) fs.ks[i] = i < nk ? ((ks[i] <= 0 || ks[i] >= V) ? V : ks[i]) : 0;
            for (int i = 0; i < kSweepMaxN; ++i) {
                if (i < nn && (ns[i] < 1 || ns[i] > kSweepMaxDrafts)) return GR_EINVAL;
                fs.ns[i] = i < nn ? ns[i] : 1;
            }
            h->solved = false;
            const int rc = prepare_full(h, B, V);
            if (rc != GR_OK) return rc;
            FullParams& f = h->full;
            f.p = p; f.q = q; f.B = B; f.V = V; f.n = 1; f.k = kmax; f.max_T = h->max_T; f.max_iter = h->max_iter;
            f.tau = 0.0; f.rel_tol = h->rel_tol; f.tail_mass = 0.0; f.logits = 0; f.temperature = nullptr; f.draft_temperature = nullptr;
            f.info = h->info; f.accept_prob = accept_prob; f.status = status; f.newton_ws = h->newton_ws;
            fs.mass = h->sweep_mass; fs.accept_prob = accept_prob; fs.status = status;
            launch_full_sweep(f, fs, stream);
            if (hipGetLastError() != hipSuccess) return GR_EHIP;
            return GR_OK;
        }
    }
    SweepParams sw;
    const int rcf = fill_sweep(sw, ks, nk, ns, nn, V);
    if (rcf != GR_OK) return rcf;
    const int splits = choose_splits(B, V);
    int slice_len = (V + splits - 1) / splits;
    slice_len = (slice_len + kSelTile - 1) / kSelTile * kSelTile;
    h->solved = false;                                   // the selection scratch of the handle is overwritten
    launch_select(p, q, B, V, sw.kmax, splits, slice_len, h->cand, h->cand_count, h->part_psum, h->part_qsum,
                  h->part_bad, h->piece_psum, h->piece_stride, stream);
    if (hipGetLastError() != hipSuccess) return GR_EHIP;
    sw.p = p; sw.splits = splits;
    sw.cand = h->cand; sw.cand_count = h->cand_count; sw.part_psum = h->part_psum; sw.part_qsum = h->part_qsum;
    sw.part_bad = h->part_bad; sw.accept_prob = accept_prob; sw.status = status;
    if (launch_sweep(sw, B, stream) != hipSuccess) return GR_EHIP;
    return GR_OK;
}

extern "C" int gr_accept_sweep_noalloc(const float* p, const float* q, const int* ks, int nk, const int* ns, int nn,
                                       int B, int V, float* accept_prob, int* status, void* hip_stream) {
    if (!p || !q || !ks || !ns || !accept_prob || !status || B <= 0 || V <= 0) return GR_EINVAL;
    if (static_cast<size_t>(B) > kNoAllocRows) return GR_ECAPACITY;
    SweepParams sw;
    const int rc = fill_sweep(sw, ks, nk, ns, nn, V);
    if (rc != GR_OK) return rc;
    unsigned char* base = nullptr;
    const int rs = scratch_address(&base);
    if (rs != GR_OK) return rs;
    unsigned long long* cand = reinterpret_cast<unsigned long long*>(base + kNaCand);
    double* psum = reinterpret_cast<double*>(base + kNaPsum);
    double* qsum = reinterpret_cast<double*>(base + kNaQsum);
    int* count = reinterpret_cast<int*>(base + kNaCount);
    int* bad = reinterpret_cast<int*>(base + kNaBad);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const int splits = choose_splits(B, V);
    int slice_len = (V + splits - 1) / splits;
    slice_len = (slice_len + kSelTile - 1) / kSelTile * kSelTile;
    launch_select(p, q, B, V, sw.kmax, splits, slice_len, cand, count, psum, qsum, bad, nullptr, 0, stream);
    if (hipGetLastError() != hipSuccess) return GR_EHIP;
    sw.p = p; sw.splits = splits;
    sw.cand = cand; sw.cand_count = count; sw.part_psum = psum; sw.part_qsum = qsum; sw.part_bad = bad;
    sw.accept_prob = accept_prob; sw.status = status;
    if (launch_sweep(sw, B, stream) != hipSuccess) return GR_EHIP;
    return GR_OK;
}

extern "C" int gr_verify(gr_handle h, const int* drafts, const float* uniforms, int* token,
                         unsigned char* accepted, void* hip_stream) {
    if (!h || !drafts || !uniforms || !token || !accepted) return GR_EINVAL;
    if (!h->solved) return GR_ESTATE;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    mark(h, 3, stream);
    launch_verify(h->p, h->B, h->V, h->n, policy_view(h), h->info, drafts, uniforms, token, accepted, stream);
    if (hipGetLastError() != hipSuccess) return GR_EHIP;
    mark(h, 4, stream);
    if (h->prof_now && h->prof_count < kProfSlots) ++h->prof_count;
    h->prof_now = false;
    return GR_OK;
}

// ---- multi-step walk over a tree of draft paths
namespace {

// dst row j = src row at element offset idx[j] (V floats), for both distributions.
__global__ __launch_bounds__(kThreads) void gather_rows_kernel(const float* __restrict__ p, const float* __restrict__ q,
                                                                const long long* __restrict__ idx, float* __restrict__ dp,
                                                                float* __restrict__ dq, int V) {
    const long long src = idx[blockIdx.x];
    const size_t dst = static_cast<size_t>(blockIdx.x) * V;
    for (int i = threadIdx.x; i < V; i += kThreads) { dp[dst + i] = p[src + i]; dq[dst + i] = q[src + i]; }
}

}  // namespace

extern "C" int gr_tree_walk(gr_handle h, const float* p, const float* q, const float* temperature, const int* paths,
                            const float* uniforms, int S, int K, int L, int V, int k, float tol,
                            int* out_tokens, int* out_len, int* out_accepted, int* out_fallbacks, void* hip_stream) {
    if (!h || !p || !q || !paths || !uniforms || !out_tokens || !out_len || !out_accepted) return GR_EINVAL;
    if (S <= 0 || K < 1 || L < 1 || V <= 0 || S > h->max_B || V > h->max_V || K > h->max_n) return GR_EINVAL;
    if (!(tol >= 0.f) || !(tol < 1.f)) return GR_EINVAL;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (!h->tw_p) {
        const size_t rows = static_cast<size_t>(h->max_B), cols = static_cast<size_t>(h->max_V);
        const bool ok = dev_alloc(&h->tw_p, rows * cols) && dev_alloc(&h->tw_q, rows * cols) && dev_alloc(&h->tw_drafts, rows * GR_MAX_N) &&
                        dev_alloc(&h->tw_u, rows) && dev_alloc(&h->tw_temp, rows) && dev_alloc(&h->tw_tok, rows) && dev_alloc(&h->tw_ok, rows) && dev_alloc(&h->tw_idx, rows) &&
                        dev_alloc(&h->tw_acc, rows) && dev_alloc(&h->tw_status, rows);
        if (!ok) {
            void* ptrs[] = {h->tw_p, h->tw_q, h->tw_drafts, h->tw_u, h->tw_temp, h->tw_tok, h->tw_ok, h->tw_idx, h->tw_acc, h->tw_status};
            for (void* ptr : ptrs) (void)hipFree(ptr);
            h->tw_p = h->tw_q = h->tw_u = h->tw_temp = h->tw_acc = nullptr; h->tw_drafts = h->tw_tok = h->tw_status = nullptr; h->tw_ok = nullptr; h->tw_idx = nullptr;
            (void)hipGetLastError();
            return GR_ENOMEM;
        }
    }
    try {
    // the state of every sequence lives on the host: the paths that still agree with the tokens emitted so far
    std::vector<unsigned> active(S, K >= 32 ? 0xFFFFFFFFu : ((1u << K) - 1u));
    std::vector<char> alive(S, 1);
    for (int s = 0; s < S; ++s) { out_len[s] = 0; out_accepted[s] = 0; if (out_fallbacks) out_fallbacks[s] = 0; }
    for (int i = 0; i < S * L; ++i) out_tokens[i] = -1;
    std::vector<int> seqs, drafts, tok, st; std::vector<long long> idx; std::vector<float> us, ts; std::vector<unsigned char> okv;
    for (int l = 0; l < L; ++l) {
        for (int n = 1; n <= K; ++n) {
            seqs.clear(); drafts.clear(); idx.clear(); us.clear(); ts.clear();
            for (int s = 0; s < S; ++s) {
                if (!alive[s] || __builtin_popcount(active[s]) != n) continue;
                const int a0 = __builtin_ctz(active[s]);
                seqs.push_back(s);
                idx.push_back(((static_cast<long long>(s) * K + a0) * L + l) * V);
                for (int a = 0; a < K; ++a) if (active[s] >> a & 1u) drafts.push_back(paths[(static_cast<size_t>(s) * K + a) * L + l]);
                us.push_back(uniforms[static_cast<size_t>(s) * L + l]);
                if (temperature) ts.push_back(temperature[s]);
            }
            const int cnt = static_cast<int>(seqs.size());
            if (cnt == 0) continue;
            if (hipMemcpyAsync(h->tw_idx, idx.data(), sizeof(long long) * cnt, hipMemcpyHostToDevice, stream) != hipSuccess ||
                hipMemcpyAsync(h->tw_drafts, drafts.data(), sizeof(int) * cnt * n, hipMemcpyHostToDevice, stream) != hipSuccess ||
                hipMemcpyAsync(h->tw_u, us.data(), sizeof(float) * cnt, hipMemcpyHostToDevice, stream) != hipSuccess ||
                (temperature && hipMemcpyAsync(h->tw_temp, ts.data(), sizeof(float) * cnt, hipMemcpyHostToDevice, stream) != hipSuccess)) return GR_EHIP;
            hipLaunchKernelGGL(gather_rows_kernel, dim3(cnt), dim3(kThreads), 0, stream, p, q, h->tw_idx, h->tw_p, h->tw_q, V);
            if (hipGetLastError() != hipSuccess) return GR_EHIP;
            const int rc = temperature
                ? gr_solve_logits_verify(h, h->tw_p, h->tw_q, h->tw_temp, nullptr, n, k, tol, cnt, V, h->tw_drafts, h->tw_u, h->tw_acc, h->tw_status,
                                         h->tw_tok, h->tw_ok, stream)
                : gr_solve_verify(h, h->tw_p, h->tw_q, n, k, tol, cnt, V, h->tw_drafts, h->tw_u, h->tw_acc, h->tw_status, h->tw_tok, h->tw_ok, stream);
            if (rc != GR_OK) return rc;
            tok.resize(cnt); st.resize(cnt); okv.resize(cnt);
            if (hipMemcpyAsync(tok.data(), h->tw_tok, sizeof(int) * cnt, hipMemcpyDeviceToHost, stream) != hipSuccess ||
                hipMemcpyAsync(okv.data(), h->tw_ok, cnt, hipMemcpyDeviceToHost, stream) != hipSuccess ||
                hipMemcpyAsync(st.data(), h->tw_status, sizeof(int) * cnt, hipMemcpyDeviceToHost, stream) != hipSuccess ||
                hipStreamSynchronize(stream) != hipSuccess) return GR_EHIP;
            for (int j = 0; j < cnt; ++j) {
                const int s = seqs[j];
                out_tokens[static_cast<size_t>(s) * L + l] = tok[j];
                out_len[s] = l + 1;
                if (out_fallbacks && st[j] != GR_ROW_OK) ++out_fallbacks[s];
                if (!okv[j] || tok[j] < 0) { alive[s] = 0; continue; }
                ++out_accepted[s];
                unsigned keep = 0u;
                for (int a = 0; a < K; ++a)
                    if ((active[s] >> a & 1u) && paths[(static_cast<size_t>(s) * K + a) * L + l] == tok[j]) keep |= 1u << a;
                active[s] = keep;
                if (!keep) alive[s] = 0;                         // cannot happen: an accepted token is one of the drafts
            }
        }
    }
    h->solved = false;                                           // the policy left in the handle belongs to a gathered batch
    return GR_OK;
    } catch (const std::bad_alloc&) {                            // host vectors: nothing may cross the C boundary
        h->solved = false;
        return GR_ENOMEM;
    }
}

extern "C" int gr_profile_stride(gr_handle h, int stride) {
    if (!h || stride < 1) return GR_EINVAL;
    if (!h->profile) return GR_ESTATE;
    h->prof_stride = stride; h->prof_tick = 0;
    return GR_OK;
}

extern "C" int gr_profile_read(gr_handle h, double* select_ms, double* solve_ms, double* verify_ms, int* steps) {
    if (!h || !select_ms || !solve_ms || !verify_ms || !steps) return GR_EINVAL;
    if (!h->profile) return GR_ESTATE;
    double acc[3] = {0.0, 0.0, 0.0};
    for (int s = 0; s < h->prof_count; ++s) {
        if (hipEventSynchronize(h->ev[s][4]) != hipSuccess) return GR_EHIP;
        const int pairs[3][2] = {{0, 1}, {1, 2}, {3, 4}};
        for (int j = 0; j < 3; ++j) {
            float ms = 0.f;
            if (hipEventElapsedTime(&ms, h->ev[s][pairs[j][0]], h->ev[s][pairs[j][1]]) != hipSuccess) return GR_EHIP;
            acc[j] += ms;
        }
    }
    const int cnt = h->prof_count;
    *steps = cnt;
    *select_ms = cnt ? acc[0] / cnt : 0.0; *solve_ms = cnt ? acc[1] / cnt : 0.0; *verify_ms = cnt ? acc[2] / cnt : 0.0;
    h->prof_count = 0;
    return GR_OK;
}

extern "C" int gr_policy_slice(gr_handle h, const int* drafts, float* pi, float* accept_given_drafts,
                               void* hip_stream) {
    if (!h || !drafts || !pi || !accept_given_drafts) return GR_EINVAL;
    if (!h->solved) return GR_ESTATE;
    launch_slice(h->p, h->B, h->V, h->n, policy_view(h), h->info, drafts, pi, accept_given_drafts,
                 static_cast<hipStream_t>(hip_stream));
    return hipGetLastError() == hipSuccess ? GR_OK : GR_EHIP;
}

namespace {

__global__ void export_kernel(const RowInfo* info, int B, int* support, int* h_size, int* iterations) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    if (support) support[b] = info[b].support;
    if (h_size) h_size[b] = info[b].h;
    if (iterations) iterations[b] = info[b].iterations;
}

__global__ void stats_kernel(const RowInfo* info, int B, int* evaluations, double* node_tokens) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    if (evaluations) evaluations[b] = info[b].iterations;
    if (node_tokens) node_tokens[b] = info[b].node_tokens;
}

}  // namespace

extern "C" int gr_policy_export(gr_handle h, int* order, int* block, double* weight, double* rho,
                                int* support, int* h_size, int* iterations, void* hip_stream) {
    if (!h) return GR_EINVAL;
    if (!h->solved) return GR_ESTATE;
    if (h->full_mode && (order || block || weight || rho)) return GR_EUNSUPPORTED;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const size_t cnt = static_cast<size_t>(h->B) * kMaxSupport;
    hipError_t e = hipSuccess;
    if (order && e == hipSuccess) e = hipMemcpyAsync(order, h->order, cnt * sizeof(int), hipMemcpyDeviceToDevice, stream);
    if (block && e == hipSuccess) e = hipMemcpyAsync(block, h->block, cnt * sizeof(int), hipMemcpyDeviceToDevice, stream);
    if (weight && e == hipSuccess) e = hipMemcpyAsync(weight, h->weight, cnt * sizeof(double), hipMemcpyDeviceToDevice, stream);
    if (rho && e == hipSuccess) e = hipMemcpyAsync(rho, h->rho, cnt * sizeof(double), hipMemcpyDeviceToDevice, stream);
    if (e != hipSuccess) return GR_EHIP;
    if (support || h_size || iterations) {
        hipLaunchKernelGGL(export_kernel, dim3((h->B + 255) / 256), dim3(256), 0, stream, h->info, h->B, support,
                           h_size, iterations);
        if (hipGetLastError() != hipSuccess) return GR_EHIP;
    }
    return GR_OK;
}

extern "C" int gr_policy_export_row(gr_handle h, int row, int count, int* order, int* block, double* weight,
                                    double* rho, void* hip_stream) {
    if (!h || row < 0 || count < 0) return GR_EINVAL;
    if (!h->solved) return GR_ESTATE;
    if (row >= h->B) return GR_EINVAL;
    const size_t stride = h->full_mode ? static_cast<size_t>(h->V) + 2 : kMaxSupport;
    if (static_cast<size_t>(count) > stride) return GR_EINVAL;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const int* s_order = h->full_mode ? h->full.order : h->order;
    const int* s_block = h->full_mode ? h->full.blk : h->block;
    const double* s_weight = h->full_mode ? h->full.weight : h->weight;
    const double* s_rho = h->full_mode ? h->full.rho : h->rho;
    const size_t off = static_cast<size_t>(row) * stride, n = static_cast<size_t>(count);
    hipError_t e = hipSuccess;
    if (n == 0) return GR_OK;
    if (order && e == hipSuccess) e = hipMemcpyAsync(order, s_order + off, n * sizeof(int), hipMemcpyDeviceToDevice, stream);
    if (block && e == hipSuccess) e = hipMemcpyAsync(block, s_block + off, n * sizeof(int), hipMemcpyDeviceToDevice, stream);
    if (weight && e == hipSuccess) e = hipMemcpyAsync(weight, s_weight + off, n * sizeof(double), hipMemcpyDeviceToDevice, stream);
    if (rho && e == hipSuccess) e = hipMemcpyAsync(rho, s_rho + off, n * sizeof(double), hipMemcpyDeviceToDevice, stream);
    return e == hipSuccess ? GR_OK : GR_EHIP;
}

extern "C" int gr_solve_stats(gr_handle h, int* evaluations, double* node_tokens, void* hip_stream) {
    if (!h) return GR_EINVAL;
    if (!h->solved) return GR_ESTATE;
    hipLaunchKernelGGL(stats_kernel, dim3((h->B + 255) / 256), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                       h->info, h->B, evaluations, node_tokens);
    return hipGetLastError() == hipSuccess ? GR_OK : GR_EHIP;
}

#ifdef GR_PHASE_CLOCKS
namespace {
__global__ void clocks_kernel(const RowInfo* info, int B, long long* out) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    for (int i = 0; i < 24; ++i) out[b * 48 + i] = info[b].clk[i];
    for (int i = 0; i < 24; ++i) out[b * 48 + 24 + i] = __double_as_longlong(info[b].errlog[i]);
}
}  // namespace
// Profiling builds only: cycles of thread 0 per phase of the last solve, [B, 48] int64 (24 cycle counts, then 24 doubles) device array.
extern "C" int gr_debug_clocks(gr_handle h, long long* out, void* hip_stream) {
    if (!h || !out || !h->solved) return GR_EINVAL;
    hipLaunchKernelGGL(clocks_kernel, dim3((h->B + 255) / 256), dim3(256), 0, static_cast<hipStream_t>(hip_stream), h->info, h->B, out);
    return hipGetLastError() == hipSuccess ? GR_OK : GR_EHIP;
}
#endif

extern "C" const char* gr_strerror(int code) {
    switch (code) {
        case GR_OK: return "ok";
        case GR_EINVAL: return "invalid argument or beyond the handle's capacity";
        case GR_ENOMEM: return "device allocation failed";
        case GR_ESTATE: return "no solved policy in this handle";
        case GR_EHIP: return "HIP runtime error";
        case GR_EUNSUPPORTED: return "a vocabulary of 2^24 tokens or more with a support above GR_MAX_SUPPORT, or a dense export of such a policy";
        case GR_ECAPACITY: return "more rows than GR_NOALLOC_MAX_B, the fixed capacity of the allocation-free entry point";
        default: return "unknown error";
    }
}
