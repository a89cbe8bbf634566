// C ABI of libmoe355 (declared in include/moe355.h): argument checks on the host, then the
// kernels of one MoE layer enqueued on the caller's stream in the order of the paper's reordered
// computation (Section 4): gate + top-k (Algorithm 1), count/offsets (Section 3.2), scatter,
// per-expert linear layers as grouped products, gather; and the reverse for the gradient.
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <vector>

#include "common.h"

namespace moe {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
}

static thread_local bool g_launch_failed = false;

void fail_launch(const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    g_launch_failed = true;
}

int current_device()
{
    int dev = -1;
    const hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        fail_launch("cannot tell the current HIP device (%s, id %d)", hipGetErrorString(e), dev);
        return -1;
    }
    return dev;
}

moe_status_t check_launch(const char* what)
{
    if (g_launch_failed) {           // the text was set by fail_launch
        g_launch_failed = false;
        (void)hipGetLastError();
        return MOE_ERR_HIP;
    }
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_error("%s: %s", what, hipGetErrorString(e));
        return MOE_ERR_HIP;
    }
    return MOE_OK;
}

// ---- optional per-kernel timing (diagnostics) --------------------------------------------------
enum Slot { S_GATE, S_PLAN, S_SCATTER, S_FC1, S_FC2, S_COMBINE, S_DCOMBINE, S_DH, S_DW2, S_DXS, S_DW1, S_GATEBWD,
            S_DH_DW2, S_DXS_DW1, S_COUNT };
static const char* const kSlotNames[S_COUNT] = {"gate_topk", "plan", "scatter", "ggemm_fc1_gelu", "ggemm_fc2",
                                                "combine", "dcombine", "ggemm_dh_dgelu", "ggemm_dw2", "ggemm_dxs",
                                                "ggemm_dw1", "gate_bwd", "ggemm_dh_dgelu+dw2", "ggemm_dxs+dw1"};
struct TimedRecord { int slot; hipEvent_t a, b; };
static std::mutex g_prof_mu;
static bool g_prof_on = false;
static std::vector<TimedRecord> g_prof_pending;
static std::vector<hipEvent_t> g_prof_pool;

static hipEvent_t prof_event()
{
    if (!g_prof_pool.empty()) { hipEvent_t e = g_prof_pool.back(); g_prof_pool.pop_back(); return e; }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

// Brackets the kernels enqueued during its lifetime with two events when profiling is on.
struct ScopedTimer {
    hipStream_t st; TimedRecord r{}; bool on = false;
    ScopedTimer(int slot, hipStream_t s) : st(s)
    {
        std::lock_guard<std::mutex> lk(g_prof_mu);
        if (!g_prof_on) return;
        r.slot = slot; r.a = prof_event(); r.b = prof_event();
        on = r.a && r.b && hipEventRecord(r.a, st) == hipSuccess;
    }
    ~ScopedTimer()
    {
        if (!on) return;
        std::lock_guard<std::mutex> lk(g_prof_mu);
        if (hipEventRecord(r.b, st) == hipSuccess) g_prof_pending.push_back(r);
    }
};

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

moe_status_t check_desc(const moe_desc_t* D)
{
    if (!D) { set_error("desc is NULL"); return MOE_ERR_INVALID_ARG; }
    if (D->N < 0 || D->d < 1 || D->h < 1 || D->E < 1 || D->k < 1 || D->k > D->E) {
        set_error("invalid sizes N=%d d=%d h=%d E=%d k=%d (need N>=0, d,h,E>=1, 1<=k<=E)", D->N, D->d, D->h, D->E, D->k);
        return MOE_ERR_INVALID_ARG;
    }
    if (D->accumulate != 0 && D->accumulate != 1) { set_error("accumulate must be 0 or 1"); return MOE_ERR_INVALID_ARG; }
    if (D->dtype != MOE_F32 && D->dtype != MOE_BF16) { set_error("unknown dtype %d", D->dtype); return MOE_ERR_UNSUPPORTED; }
    if (D->grad_dtype != D->dtype && D->grad_dtype != MOE_F32) {
        set_error("grad_dtype %d unsupported with dtype %d (must equal dtype or be fp32)", D->grad_dtype, D->dtype);
        return MOE_ERR_UNSUPPORTED;
    }
    if (D->d % 32 || D->h % 32) { set_error("d=%d and h=%d must be multiples of 32", D->d, D->h); return MOE_ERR_UNSUPPORTED; }
    if (D->E > kMaxE) { set_error("E=%d exceeds %d", D->E, kMaxE); return MOE_ERR_UNSUPPORTED; }
    if (D->k > kMaxK) { set_error("k=%d exceeds %d", D->k, kMaxK); return MOE_ERR_UNSUPPORTED; }
    if (D->score_all != 0 && D->score_all != 1) { set_error("score_all must be 0 or 1"); return MOE_ERR_INVALID_ARG; }
    if (D->balance_stats != 0 && D->balance_stats != 1) { set_error("balance_stats must be 0 or 1"); return MOE_ERR_INVALID_ARG; }
    for (int i = 0; i < 6; ++i)
        if (D->reserved[i]) { set_error("reserved[%d] must be 0", i); return MOE_ERR_UNSUPPORTED; }
    const long long M = (long long)D->N * D->k;
    if (M > 0x7fffffffLL || M * (long long)(D->d > D->h ? D->d : D->h) > (1LL << 46)) {
        set_error("problem too large: N*k=%lld", M);
        return MOE_ERR_UNSUPPORTED;
    }
    return MOE_OK;
}

#define MOE_REQUIRE_PTR(p)                                                               \
    do {                                                                                 \
        if (!(p)) { set_error(#p " is NULL"); return MOE_ERR_INVALID_ARG; }              \
        if (!aligned16(p)) { set_error(#p " is not 16-byte aligned"); return MOE_ERR_INVALID_ARG; } \
    } while (0)

static moe_status_t check_plan(const moe_plan_t* P)
{
    if (!P) { set_error("plan is NULL"); return MOE_ERR_INVALID_ARG; }
    MOE_REQUIRE_PTR(P->topk_idx);
    MOE_REQUIRE_PTR(P->topk_w);
    MOE_REQUIRE_PTR(P->counts);
    MOE_REQUIRE_PTR(P->offsets);
    MOE_REQUIRE_PTR(P->pos);
    MOE_REQUIRE_PTR(P->perm);
    return MOE_OK;
}

static moe_status_t check_ws(const moe_desc_t* D, const void* ws, size_t bytes, WsLayout* L)
{
    MOE_REQUIRE_PTR(ws);
    *L = ws_layout(*D);
    if (bytes < L->total) {
        set_error("workspace too small: %zu bytes given, %zu needed", bytes, L->total);
        return MOE_ERR_WORKSPACE;
    }
    return MOE_OK;
}

// Top-1 with the score fixed at 1: moe_forward writes Y from the second layer and keeps no Ys.
static bool direct_top1(const moe_desc_t& D) { return D.k == 1 && !D.score_all; }

static void run_gemm(const moe_desc_t& D, GemmArgs& a, hipStream_t st)
{
    if (D.dtype == MOE_BF16) launch_ggemm_bf16_sk(a, st);
    else launch_ggemm_f32(a, st);
}

}  // namespace moe

using namespace moe;

extern "C" {

size_t moe_workspace_bytes(const moe_desc_t* desc)
{
    if (check_desc(desc) != MOE_OK) return 0;
    return ws_layout(*desc).total;
}

const char* moe_last_error(void) { return g_err; }

moe_status_t moe_profile_enable(int on)
{
    std::lock_guard<std::mutex> lk(g_prof_mu);
    for (auto& r : g_prof_pending) { g_prof_pool.push_back(r.a); g_prof_pool.push_back(r.b); }
    g_prof_pending.clear();
    g_prof_on = on != 0;
    return MOE_OK;
}

int moe_profile_read(moe_kernel_time_t* out, int max_entries)
{
    g_err[0] = 0;
    if (!out || max_entries < 0) { set_error("out is NULL or max_entries < 0"); return MOE_ERR_INVALID_ARG; }
    std::lock_guard<std::mutex> lk(g_prof_mu);
    int launches[S_COUNT] = {};
    double ms[S_COUNT] = {};
    int rc = 0;
    for (auto& r : g_prof_pending) {
        float t = 0.f;
        if (hipEventSynchronize(r.b) != hipSuccess || hipEventElapsedTime(&t, r.a, r.b) != hipSuccess) {
            set_error("profile: %s", hipGetErrorString(hipGetLastError()));
            rc = MOE_ERR_HIP;
        }
        launches[r.slot] += 1;
        ms[r.slot] += t;
        g_prof_pool.push_back(r.a);
        g_prof_pool.push_back(r.b);
    }
    g_prof_pending.clear();
    if (rc) return rc;
    int n = 0;
    for (int s = 0; s < S_COUNT && n < max_entries; ++s)
        if (launches[s]) out[n++] = moe_kernel_time_t{kSlotNames[s], launches[s], ms[s]};
    return n;
}

moe_status_t moe_workspace_region(const moe_desc_t* desc, const char* name, size_t* offset, size_t* bytes)
{
    g_err[0] = 0;
    moe_status_t s;
    if ((s = check_desc(desc)) != MOE_OK) return s;
    if (!name || !offset || !bytes) { set_error("name, offset and bytes must not be NULL"); return MOE_ERR_INVALID_ARG; }
    const WsLayout L = ws_layout(*desc);
    const size_t M = (size_t)desc->N * desc->k, b = dtype_size(desc->dtype);
    const struct { const char* n; size_t off, len; } regions[] = {
        {"Xs", L.Xs, M * desc->d * b}, {"Z", L.Z, M * desc->h * b},     {"H", L.H, M * desc->h * b},
        {"Ys", L.Ys, M * desc->d * b}, {"dYs", L.dYs, M * desc->d * b}, {"dZ", L.dZ, M * desc->h * b},
        {"dXs", L.dXs, M * desc->d * b}, {"dl", L.dl, M * sizeof(float)},
        {"gate_uncertified", L.gate_fail, ((size_t)desc->N + 1) * sizeof(int32_t)},
        {"status", L.sk_error, sizeof(int32_t)},
        {"clock", L.zeros + kCtlClock * sizeof(int32_t), 2 * sizeof(long long)},
    };
    for (const auto& r : regions)
        if (!strcmp(r.n, name)) { *offset = r.off; *bytes = r.len; return MOE_OK; }
    set_error("unknown workspace region '%s'", name);
    return MOE_ERR_INVALID_ARG;
}

moe_status_t moe_check_status(const moe_desc_t* desc, const void* workspace, size_t workspace_bytes, void* stream,
                              int32_t* status)
{
    g_err[0] = 0;
    moe_status_t s;
    if ((s = check_desc(desc)) != MOE_OK) return s;
    if (!status) { set_error("status is NULL"); return MOE_ERR_INVALID_ARG; }
    WsLayout L;
    if ((s = check_ws(desc, workspace, workspace_bytes, &L)) != MOE_OK) return s;
    hipError_t e = hipStreamSynchronize((hipStream_t)stream);
    if (e == hipSuccess) e = hipMemcpy(status, (const char*)workspace + L.sk_error, sizeof(int32_t), hipMemcpyDeviceToHost);
    if (e != hipSuccess) { set_error("moe_check_status: %s", hipGetErrorString(e)); return MOE_ERR_HIP; }
    if (*status) set_error("a grouped-product workgroup's bounded wait for a partial sum ran out: the results of the calls on this workspace since the last moe_plan are invalid");
    return MOE_OK;
}

moe_status_t moe_plan(const moe_desc_t* desc, const void* X, const void* Wg, const float* bg, moe_plan_t* plan,
                      void* workspace, size_t workspace_bytes, void* stream)
{
    g_err[0] = 0;
    moe_status_t s;
    if ((s = check_desc(desc)) != MOE_OK) return s;
    if ((s = check_plan(plan)) != MOE_OK) return s;
    MOE_REQUIRE_PTR(X);
    MOE_REQUIRE_PTR(Wg);
    if (bg && (reinterpret_cast<uintptr_t>(bg) & 3u)) { set_error("bg is not 4-byte aligned"); return MOE_ERR_INVALID_ARG; }
    WsLayout L;
    if ((s = check_ws(desc, workspace, workspace_bytes, &L)) != MOE_OK) return s;
    hipStream_t st = (hipStream_t)stream;
    const moe_desc_t& D = *desc;
    if (D.N > 0) {
        ScopedTimer tm(S_GATE, st);
        launch_gate_topk(D, X, Wg, bg, plan->topk_idx, plan->topk_w, (char*)workspace + L.WgT,
                         (D.score_all || D.balance_stats) ? (double*)((char*)workspace + L.logits) : nullptr,
                         (D.score_all || D.balance_stats) ? (double*)((char*)workspace + L.lse) : nullptr,
                         (int32_t*)((char*)workspace + L.gate_fail), st);
        if ((s = check_launch("gate/top-k")) != MOE_OK) return s;
    }
    // With N == 0 the plan kernels still run: they write counts = 0, offsets = 0 and empty tile tables.
    {
        ScopedTimer tm(S_PLAN, st);
        launch_plan(D, L, plan->topk_idx, plan->counts, plan->offsets, plan->pos, plan->perm, (char*)workspace, st);
    }
    return check_launch("plan");
}

moe_status_t moe_forward(const moe_desc_t* desc, const moe_plan_t* plan, const void* X, const void* W1,
                         const void* W2, const void* b1, const void* b2, void* Y, void* workspace,
                         size_t workspace_bytes, void* stream)
{
    g_err[0] = 0;
    moe_status_t s;
    if ((s = check_desc(desc)) != MOE_OK) return s;
    if ((s = check_plan(plan)) != MOE_OK) return s;
    MOE_REQUIRE_PTR(X);
    MOE_REQUIRE_PTR(W1);
    MOE_REQUIRE_PTR(W2);
    if (b1 && !aligned16(b1)) { set_error("b1 is not 16-byte aligned"); return MOE_ERR_INVALID_ARG; }
    if (b2 && !aligned16(b2)) { set_error("b2 is not 16-byte aligned"); return MOE_ERR_INVALID_ARG; }
    WsLayout L;
    if ((s = check_ws(desc, workspace, workspace_bytes, &L)) != MOE_OK) return s;
    const moe_desc_t& D = *desc;
    if (D.N == 0) return MOE_OK;
    MOE_REQUIRE_PTR(Y);
    hipStream_t st = (hipStream_t)stream;
    char* ws = (char*)workspace;

    // No scatter launch here: the first layer fetches row perm[r] / k of X as row r of its operand, which is the
    // scatter of Section 4 done on the fly (moe_backward writes Xs when the weight gradient needs it).
    GemmArgs a{};
    a.M = (long)D.N * D.k;
    a.stream_out = (size_t)D.E * D.d * D.h * 2 > ((size_t)48 << 20);   // (the experts' weights do not fit the L2 caches: see store_out)
    a.E = D.E;
    a.counts = plan->counts;
    a.offsets = plan->offsets;
    a.tileP = (const int32_t*)(ws + L.tileP);
    a.order = (const int32_t*)(ws + L.order);
    a.cls = (const int32_t*)(ws + L.cls);
    set_control(a, ws, L);

    a.kind = kRowsNN_GeLU;  // Z = Xs W1[e],  H = GeLU(Z)
    a.A = X; a.a_gather = plan->perm; a.a_gather_div = D.k;
    a.B = W1; a.C = ws + L.Z; a.C2 = ws + L.H; a.K = D.d; a.Nout = D.h; a.bias = b1;
    { ScopedTimer tm(S_FC1, st); run_gemm(D, a, st); }
    if ((s = check_launch("expert layer 1")) != MOE_OK) return s;

    a.kind = kRowsNN;       // Ys = H W2[e]
    a.A = ws + L.H; a.a_gather = nullptr; a.B = W2; a.C = ws + L.Ys; a.C2 = nullptr; a.K = D.h; a.Nout = D.d; a.bias = b2;
    // Top-1 with the score fixed at 1 (softmax over one logit): y is the one expert's output, so the second layer
    // writes row r straight to Y[perm[r]] - the gather of Section 4 done on the fly; Ys is not written.
    const bool direct = direct_top1(D);
    if (direct) { a.C = Y; a.c_scatter = plan->perm; }
    { ScopedTimer tm(S_FC2, st); run_gemm(D, a, st); }
    if ((s = check_launch("expert layer 2")) != MOE_OK) return s;
    if (direct) return MOE_OK;

    { ScopedTimer tm(S_COMBINE, st); launch_combine(D, ws + L.Ys, plan->topk_w, plan->pos, Y, st); }
    return check_launch("combine");
}

moe_status_t moe_backward(const moe_desc_t* desc, const moe_plan_t* plan, const void* X, const void* Wg,
                          const void* W1, const void* W2, const void* dY, void* dX, void* dWg, float* dbg,
                          void* dW1, void* dW2, void* workspace, size_t workspace_bytes, void* stream)
{
    g_err[0] = 0;
    moe_status_t s;
    if ((s = check_desc(desc)) != MOE_OK) return s;
    if ((s = check_plan(plan)) != MOE_OK) return s;
    MOE_REQUIRE_PTR(X);
    MOE_REQUIRE_PTR(Wg);
    MOE_REQUIRE_PTR(W1);
    MOE_REQUIRE_PTR(W2);
    MOE_REQUIRE_PTR(dWg);
    MOE_REQUIRE_PTR(dW1);
    MOE_REQUIRE_PTR(dW2);
    if (dbg && (reinterpret_cast<uintptr_t>(dbg) & 3u)) { set_error("dbg is not 4-byte aligned"); return MOE_ERR_INVALID_ARG; }
    WsLayout L;
    if ((s = check_ws(desc, workspace, workspace_bytes, &L)) != MOE_OK) return s;
    const moe_desc_t& D = *desc;
    if (D.N > 0) {
        MOE_REQUIRE_PTR(dY);
        MOE_REQUIRE_PTR(dX);
    }
    hipStream_t st = (hipStream_t)stream;
    char* ws = (char*)workspace;

    if (D.N > 0) {
        // The same launch writes Xs for the first layer's weight gradient and the gate's (the forward pass read X
        // through perm instead).
        ScopedTimer tm(S_DCOMBINE, st);
        launch_dcombine(D, dY, direct_top1(D) ? nullptr : ws + L.Ys, plan->topk_w, plan->pos, ws + L.dYs, (float*)(ws + L.dl),
                        D.score_all ? (float*)(ws + L.gate_S) : nullptr, X, ws + L.Xs, st);
        if ((s = check_launch("combine backward")) != MOE_OK) return s;
    }

    GemmArgs a{};
    a.M = (long)D.N * D.k;
    a.stream_out = (size_t)D.E * D.d * D.h * 2 > ((size_t)48 << 20);   // (the experts' weights do not fit the L2 caches: see store_out)
    a.E = D.E;
    a.counts = plan->counts;
    a.offsets = plan->offsets;
    a.tileP = (const int32_t*)(ws + L.tileP);
    a.order = (const int32_t*)(ws + L.order);
    a.cls = (const int32_t*)(ws + L.cls);
    set_control(a, ws, L);
    a.out_f32 = D.grad_dtype == MOE_F32;
    a.accumulate = D.accumulate;

    GemmArgs dh = a, dw2 = a, dxs = a, dw1 = a;
    dh.kind = kRowsNT_dGeLU;     // dZ = (dYs W2[e]^T) .* GeLU'(Z)
    dh.A = ws + L.dYs; dh.B = W2; dh.C = ws + L.dZ; dh.Zin = ws + L.Z; dh.K = D.d; dh.Nout = D.h;
    dw2.kind = kColsT;           // dW2[e] = H[seg]^T dYs[seg]
    dw2.A = ws + L.H; dw2.B = ws + L.dYs; dw2.C = dW2; dw2.K = D.h; dw2.Nout = D.d;
    dxs.kind = kRowsNT;          // dXs = dZ W1[e]^T
    dxs.A = ws + L.dZ; dxs.B = W1; dxs.C = ws + L.dXs; dxs.K = D.h; dxs.Nout = D.d;
    dw1.kind = kColsT;           // dW1[e] = Xs[seg]^T dZ[seg]
    dw1.A = ws + L.Xs; dw1.B = ws + L.dZ; dw1.C = dW1; dw1.K = D.d; dw1.Nout = D.h;
    // dZ and dW2 need only dYs, and dXs and dW1 only dZ: where it pays, each pair is one launch in which a workgroup
    // that has finished its share of the first product goes on with tiles of the second.
    const bool can_pair = D.dtype == MOE_BF16 && D.N > 0;
    if (can_pair && ggemm_pair_pays(dh)) {
        { ScopedTimer tm(S_DH_DW2, st); launch_ggemm_pair_bf16_sk(dh, dw2, st); }
        if ((s = check_launch("expert layer 2 gradients")) != MOE_OK) return s;
    } else {
        if (D.N > 0) {
            { ScopedTimer tm(S_DH, st); run_gemm(D, dh, st); }
            if ((s = check_launch("expert layer 2 data gradient")) != MOE_OK) return s;
        }
        // The weight-gradient launches also run for N == 0: they write zeros (or leave the buffers when accumulating).
        { ScopedTimer tm(S_DW2, st); run_gemm(D, dw2, st); }
        if ((s = check_launch("expert layer 2 weight gradient")) != MOE_OK) return s;
    }
    if (can_pair && ggemm_pair_pays(dxs)) {
        { ScopedTimer tm(S_DXS_DW1, st); launch_ggemm_pair_bf16_sk(dxs, dw1, st); }
        if ((s = check_launch("expert layer 1 gradients")) != MOE_OK) return s;
    } else {
        if (D.N > 0) {
            { ScopedTimer tm(S_DXS, st); run_gemm(D, dxs, st); }
            if ((s = check_launch("expert layer 1 data gradient")) != MOE_OK) return s;
        }
        { ScopedTimer tm(S_DW1, st); run_gemm(D, dw1, st); }
        if ((s = check_launch("expert layer 1 weight gradient")) != MOE_OK) return s;
    }

    {
        ScopedTimer tm(S_GATEBWD, st);
        launch_gate_bwd(D, L, ws + L.Xs, ws + L.dXs, Wg, (const float*)(ws + L.dl), plan->topk_idx, plan->pos,
                        plan->perm, plan->counts, plan->offsets, dX, dWg, dbg, ws, D.score_all ? X : nullptr, st);
    }
    return check_launch("gate backward");
}

moe_status_t moe_balance_stats(const moe_desc_t* desc, const moe_plan_t* plan, float* fraction, float* mean_prob,
                               float* loss, void* workspace, size_t workspace_bytes, void* stream)
{
    g_err[0] = 0;
    moe_status_t s;
    if ((s = check_desc(desc)) != MOE_OK) return s;
    if ((s = check_plan(plan)) != MOE_OK) return s;
    if (!desc->balance_stats && !desc->score_all) {
        set_error("moe_balance_stats needs desc.balance_stats or desc.score_all (moe_plan keeps the gate logits only then)");
        return MOE_ERR_UNSUPPORTED;
    }
    for (const float* p : {fraction, mean_prob, loss})
        if (p && (reinterpret_cast<uintptr_t>(p) & 3u)) { set_error("output is not 4-byte aligned"); return MOE_ERR_INVALID_ARG; }
    WsLayout L;
    if ((s = check_ws(desc, workspace, workspace_bytes, &L)) != MOE_OK) return s;
    launch_balance_stats(*desc, L, plan->counts, fraction, mean_prob, loss, (char*)workspace, (hipStream_t)stream);
    return check_launch("balance statistics");
}

moe_status_t moe_bias_backward(const moe_desc_t* desc, const moe_plan_t* plan, float* db1, float* db2, void* workspace,
                               size_t workspace_bytes, void* stream)
{
    g_err[0] = 0;
    moe_status_t s;
    if ((s = check_desc(desc)) != MOE_OK) return s;
    if ((s = check_plan(plan)) != MOE_OK) return s;
    if (db1 && !aligned16(db1)) { set_error("db1 is not 16-byte aligned"); return MOE_ERR_INVALID_ARG; }
    if (db2 && !aligned16(db2)) { set_error("db2 is not 16-byte aligned"); return MOE_ERR_INVALID_ARG; }
    WsLayout L;
    if ((s = check_ws(desc, workspace, workspace_bytes, &L)) != MOE_OK) return s;
    const moe_desc_t& D = *desc;
    hipStream_t st = (hipStream_t)stream;
    char* ws = (char*)workspace;
    // z = xs W1 + b1 and ys = h W2 + b2 per row: the bias gradients are the column sums, over the expert's rows,
    // of dZ and of dYs, which moe_backward left in the workspace.  (With N == 0 every sum is empty.)
    if (db1) launch_segment_sums(D, L, ws + L.dZ, D.h, plan->counts, plan->offsets, db1, ws, st);
    if (db2) launch_segment_sums(D, L, ws + L.dYs, D.d, plan->counts, plan->offsets, db2, ws, st);
    return check_launch("expert bias gradients");
}

moe_status_t moe_scatter(const moe_desc_t* desc, const moe_plan_t* plan, const void* X, void* Xs, void* stream)
{
    g_err[0] = 0;
    moe_status_t s;
    if ((s = check_desc(desc)) != MOE_OK) return s;
    if ((s = check_plan(plan)) != MOE_OK) return s;
    MOE_REQUIRE_PTR(X);
    MOE_REQUIRE_PTR(Xs);
    if (desc->N == 0) return MOE_OK;
    launch_scatter(*desc, X, plan->perm, Xs, (hipStream_t)stream);
    return check_launch("scatter");
}

moe_status_t moe_gather(const moe_desc_t* desc, const moe_plan_t* plan, const void* Ys, void* Y, void* stream)
{
    g_err[0] = 0;
    moe_status_t s;
    if ((s = check_desc(desc)) != MOE_OK) return s;
    if ((s = check_plan(plan)) != MOE_OK) return s;
    MOE_REQUIRE_PTR(Ys);
    MOE_REQUIRE_PTR(Y);
    if (desc->N == 0) return MOE_OK;
    launch_combine(*desc, Ys, plan->topk_w, plan->pos, Y, (hipStream_t)stream);
    return check_launch("gather");
}

moe_status_t moe_gather_backward(const moe_desc_t* desc, const moe_plan_t* plan, const void* dY, const void* Ys,
                                 void* dYs, float* dl, void* stream)
{
    g_err[0] = 0;
    moe_status_t s;
    if ((s = check_desc(desc)) != MOE_OK) return s;
    if ((s = check_plan(plan)) != MOE_OK) return s;
    MOE_REQUIRE_PTR(dY);
    MOE_REQUIRE_PTR(Ys);
    MOE_REQUIRE_PTR(dYs);
    if (!dl || (reinterpret_cast<uintptr_t>(dl) & 3u)) { set_error("dl is NULL or not 4-byte aligned"); return MOE_ERR_INVALID_ARG; }
    if (desc->score_all) { set_error("moe_gather_backward / moe_scatter_backward carry the gradient of the selected experts only (score_all must be 0)"); return MOE_ERR_UNSUPPORTED; }
    if (desc->N == 0) return MOE_OK;
    launch_dcombine(*desc, dY, Ys, plan->topk_w, plan->pos, dYs, dl, nullptr, nullptr, nullptr, (hipStream_t)stream);
    return check_launch("gather backward");
}

moe_status_t moe_scatter_backward(const moe_desc_t* desc, const moe_plan_t* plan, const void* Wg, const void* Xs,
                                  const void* dXs, const float* dl, void* dX, void* dWg, float* dbg,
                                  void* workspace, size_t workspace_bytes, void* stream)
{
    g_err[0] = 0;
    moe_status_t s;
    if ((s = check_desc(desc)) != MOE_OK) return s;
    if ((s = check_plan(plan)) != MOE_OK) return s;
    MOE_REQUIRE_PTR(Wg);
    MOE_REQUIRE_PTR(dWg);
    if (dbg && (reinterpret_cast<uintptr_t>(dbg) & 3u)) { set_error("dbg is not 4-byte aligned"); return MOE_ERR_INVALID_ARG; }
    WsLayout L;
    if ((s = check_ws(desc, workspace, workspace_bytes, &L)) != MOE_OK) return s;
    if (desc->N > 0) {
        MOE_REQUIRE_PTR(Xs);
        MOE_REQUIRE_PTR(dXs);
        MOE_REQUIRE_PTR(dX);
        if (!dl || (reinterpret_cast<uintptr_t>(dl) & 3u)) { set_error("dl is NULL or not 4-byte aligned"); return MOE_ERR_INVALID_ARG; }
    }
    if (desc->score_all) { set_error("moe_gather_backward / moe_scatter_backward carry the gradient of the selected experts only (score_all must be 0)"); return MOE_ERR_UNSUPPORTED; }
    launch_gate_bwd(*desc, L, Xs, dXs, Wg, dl, plan->topk_idx, plan->pos, plan->perm, plan->counts, plan->offsets, dX,
                    dWg, dbg, (char*)workspace, nullptr, (hipStream_t)stream);
    return check_launch("scatter backward");
}

}  // extern "C"
