// moe_scatter_backward_static: moe_scatter_backward for callers that cannot allocate device memory (code under
// HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).  The kernels and their order are
// those of moe_scatter_backward; what that call keeps in the caller's workspace -- the 64-row piece table, the
// fp32 partial sums of the gate-matrix gradient and the transposed gate matrix -- lives here in a file-scope
// device array of fixed size instead.  Every GPU the library runs on holds its own copy of the array at its own
// address until the process ends; the address is looked up once per device, with that device current.
#include <mutex>

#include "common.h"

namespace moe {

constexpr size_t kStaticScratchBytes = 16u << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

static std::mutex g_scratch_mu;
static void* g_scratch_ptr[kMaxDevices] = {};

// Device address of this device's copy of the array (nullptr and an error text on failure).
static char* static_scratch()
{
    const int dev = current_device();
    if (dev < 0) return nullptr;
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            fail_launch("static scratch: hipGetSymbolAddress failed: %s", hipGetErrorString(e));
            return nullptr;
        }
        g_scratch_ptr[dev] = p;
    }
    return (char*)g_scratch_ptr[dev];
}

// P[e] = number of 64-row pieces of the experts before e, P[E] = their total (one workgroup; E <= 1024).
__global__ __launch_bounds__(1024) void piece_prefix_64(const int32_t* __restrict__ counts, int E, int32_t* __restrict__ P)
{
    __shared__ int s[kMaxE];
    const int e = threadIdx.x;
    s[e] = e < E ? (counts[e] + 63) / 64 : 0;
    __syncthreads();
    for (int off = 1; off < kMaxE; off <<= 1) {
        const int v = e >= off ? s[e - off] : 0;
        __syncthreads();
        s[e] += v;
        __syncthreads();
    }
    if (e < E) P[e + 1] = s[e];
    if (e == 0) P[0] = 0;
}

}  // namespace moe

using namespace moe;

extern "C" moe_status_t moe_scatter_backward_static(const moe_desc_t* desc, const moe_plan_t* plan, const void* Wg,
                                                    const void* Xs, const void* dXs, const float* dl, void* dX,
                                                    void* dWg, float* dbg, void* stream)
{
    set_error("%s", "");
    moe_status_t s;
    if ((s = check_desc(desc)) != MOE_OK) return s;
    if (!plan) { set_error("plan is NULL"); return MOE_ERR_INVALID_ARG; }
    const moe_desc_t& D = *desc;
    if (D.score_all) { set_error("moe_scatter_backward_static carries the gradient of the selected experts only (score_all must be 0)"); return MOE_ERR_UNSUPPORTED; }
    auto bad = [](const void* p, unsigned mask) { return !p || (reinterpret_cast<uintptr_t>(p) & mask); };
    if (bad(plan->topk_idx, 15) || bad(plan->counts, 15) || bad(plan->offsets, 15) || bad(plan->pos, 15) || bad(plan->perm, 15)) {
        set_error("a plan array is NULL or not 16-byte aligned");
        return MOE_ERR_INVALID_ARG;
    }
    if (bad(Wg, 15) || bad(dWg, 15) || (dbg && bad(dbg, 3))) { set_error("Wg / dWg is NULL or misaligned, or dbg is misaligned"); return MOE_ERR_INVALID_ARG; }
    if (D.N > 0 && (bad(Xs, 15) || bad(dXs, 15) || bad(dX, 15) || bad(dl, 3))) {
        set_error("Xs, dXs, dX or dl is NULL or misaligned");
        return MOE_ERR_INVALID_ARG;
    }
    // layout inside the array: the four-height piece table of launch_gate_bwd (only the 64-row line is filled),
    // partial sums of dWg and dbg by piece, the transposed gate matrix
    const size_t M = (size_t)D.N * D.k;
    WsLayout L{};
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes, 256); return at; };
    L.tileP = take((size_t)kNumTileHeights * (D.E + 1) * sizeof(int32_t));
    L.dwg_pieces = (long)(M / 64) + D.E;
    L.dwg_part = take((size_t)L.dwg_pieces * D.d * sizeof(float));
    L.dbg_part = take((size_t)L.dwg_pieces * sizeof(float));
    L.WgT = take((size_t)D.E * D.d * dtype_size(D.dtype));
    L.total = o;
    if (L.total > kStaticScratchBytes) {
        set_error("moe_scatter_backward_static: this problem needs %zu bytes of scratch, the fixed array holds %zu "
                  "(about (N k / 64 + E) d 4 bytes); use moe_scatter_backward with a workspace",
                  L.total, kStaticScratchBytes);
        return MOE_ERR_WORKSPACE;
    }
    char* const ws = static_scratch();
    if (!ws) return check_launch("static scratch");
    hipStream_t st = (hipStream_t)stream;
    int32_t* P64 = (int32_t*)(ws + L.tileP) + tile_height_index(64) * (D.E + 1);
    hipLaunchKernelGGL(piece_prefix_64, dim3(1), dim3(1024), 0, st, (const int32_t*)plan->counts, D.E, P64);
    launch_gate_bwd(D, L, Xs, dXs, Wg, dl, plan->topk_idx, plan->pos, plan->perm, plan->counts, plan->offsets, dX, dWg, dbg,
                    ws, nullptr, st);
    return check_launch("scatter backward (static scratch)");
}
