// Shared host/device declarations of libmoe355 (internal; the public ABI is include/moe355.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <mutex>

#include "../../include/moe355.h"

namespace moe {

constexpr int kMaxE = 1024;
constexpr int kMaxK = 8;
constexpr int kPlanChunk = 1024;  // assignments ranked by one workgroup of the plan kernels
constexpr int kNumTileHeights = 4;  // row-tile prefix tables are kept for 32, 64, 128, 256 rows
constexpr int kMaxPersistentWgs = 256;               // persistent grouped-GEMM workgroups (one per compute unit)
constexpr size_t kPartialBytesPerWg = 256 * 256 * 4;  // one fp32 output tile of partial sums per workgroup
// Size classes of an expert's rows for the bf16 row products: whole blocks of kClsBigRows rows, computed in
// 256 x 256 tiles, and a last piece of at most kClsSmallRows rows, computed in 128 x 512 tiles (half as many tiles
// for it).  A last piece longer than that counts as one more big block.  Tables, each [E+1]:
constexpr int kClsBigRows = 256, kClsSmallRows = 128;
enum { kClsCountsBig = 0,    // rows of the expert that the big tiles cover
       kClsCountsSmall = 1,  // rows of its last piece (0: none)
       kClsOffsetsSmall = 2, // first row of the last piece
       kClsPBig = 3,         // prefix of the number of big row blocks ([E] = total)
       kClsPSmall = 4,       // prefix of the number of last pieces ([E] = total)
       kClsTables = 5 };
__host__ __device__ constexpr int tile_height(int q) { return 32 << q; }
__host__ __device__ constexpr int tile_height_index(int bm) { return bm == 32 ? 0 : bm == 64 ? 1 : bm == 128 ? 2 : 3; }

// ---- workspace layout (byte offsets from the workspace base; every region 256-B aligned) ----
struct WsLayout {
    size_t Xs, Z, H, Ys, dYs, dZ, dXs;  // expert-contiguous activations / gradients, element type = desc.dtype
    size_t dl;        // [M]  float: gradient of the selected logits, by assignment
    size_t tileP;     // [4][E+1] int32: prefix of ceil(counts/BM) for BM = 32,64,128,256
    size_t order;     // [E] int32: experts by descending count (ties: lower id first)
    size_t cls;       // [5][E+1] int32: the experts' rows in two size classes (see kCls* below)
    size_t hist;      // [nb][E] int32: per plan-chunk histogram, then exclusive base inside the expert
    size_t dwg_part;  // [pieces][d] float: partial sums of dWg over pieces of 64 rows
    size_t dbg_part;  // [pieces] float
    size_t bias_part; // [pieces][max(d,h)] float: partial column sums for the expert-bias gradients
    // only with desc.score_all or desc.balance_stats:
    size_t logits;    // [N][E] double: the gate logits
    size_t lse;       // [N] double: log of the sum of exp of a token's logits
    size_t prob_part; // [ceil(N/512)][E] double: sums of the gate probabilities by chunk of 512 tokens
    // only with desc.score_all (scores = softmax over all experts):
    size_t gate_S;    // [N] float: sum_j w_j dL/dw_j of a token
    size_t gate_R;    // [N][E] float: dL/dlogit of the experts that were not selected (0 at the selected ones)
    size_t dx_dense;  // [N][d] float: their contribution to dX
    size_t dense_part;   // [ceil(N/512)][E][d] float: their contribution to dWg, by chunk of 512 tokens
    size_t dense_bpart;  // [ceil(N/512)][E] float: and to dbg
    int dense_chunks;
    size_t gate_fail; // [1 + N] int32: how many tokens the fast gate kernel could not certify, then their ids
    size_t WgT;       // [E][d] gate matrix transposed (written by the plan step for E > 32 and by the backward pass), element type = desc.dtype
    size_t zeros;     // the control block (see Ctl below): 1 KB of zeros, source of masked reduction rows, then the control words
    size_t sk_flags;  // [kSkPhases][kMaxPersistentWgs] int32 "partial sum ready", zeroed with the zero page
    size_t sk_error;  // int32: set if a wait for a partial sum ran out
    size_t sk_part;   // [kSkPhases][kMaxPersistentWgs] fp32 tiles: partial sums of split output tiles (bf16 only)
    size_t total;
    int nb;           // plan chunks = ceil(M / kPlanChunk)
    long dwg_pieces;  // upper bound of 64-row pieces over all experts: floor(M/64) + E
};

// A launch may run two products' worth of split tiles one after the other (the two size classes of the rows
// kinds): each phase has partial-sum buffers and flags of its own, so a workgroup that is already in the second
// phase never overwrites a partial sum of the first that its successor has not read yet.
constexpr int kSkPhases = 2;
// The control block of a workspace, in int32 words from its start.  The plan step zeroes all of it and then sets
// by_expert and skewed; the grouped products read and update the rest.
enum Ctl {
    kCtlZeroPage = 0,                                          // 256 words of zeros
    kCtlFlags = 256,                                           // [kSkPhases][kMaxPersistentWgs] "partial sum ready"
    kCtlError = kCtlFlags + kSkPhases * kMaxPersistentWgs,     // status word: 1 if a bounded wait ran out
    kCtlByExpert = kCtlError + 1,                              // 1: the weight gradients give every XCD whole experts
    kCtlClock = kCtlError + 2,                                 // two int64: shader cycles, 100 MHz ticks (8-byte aligned)
    kCtlSkewed = kCtlError + 6,                                // 1: the experts' sizes are strongly skewed
    kCtlDyn = kCtlError + 8,                                   // [9] on-demand tile counters per XCD + workgroups finished
    kCtlWords = kCtlError + 32
};
static_assert(kCtlClock % 2 == 0 && kCtlWords <= 1024, "clock words 8-byte aligned; one 1024-thread workgroup zeroes the block");
constexpr size_t kZeroedBytes = kCtlWords * sizeof(int32_t);
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline size_t dtype_size(int dt) { return dt == MOE_BF16 ? 2 : 4; }

inline WsLayout ws_layout(const moe_desc_t& D)
{
    WsLayout L{};
    const size_t M = (size_t)D.N * D.k, b = dtype_size(D.dtype);
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes, 256); return at; };
    L.Xs = take(M * D.d * b);
    L.Z = take(M * D.h * b);
    L.H = take(M * D.h * b);
    L.Ys = take(M * D.d * b);
    L.dYs = take(M * D.d * b);
    L.dZ = take(M * D.h * b);
    L.dXs = take(M * D.d * b);
    L.dl = take(M * sizeof(float));
    L.tileP = take((size_t)kNumTileHeights * (D.E + 1) * sizeof(int32_t));
    L.order = take((size_t)D.E * sizeof(int32_t));
    L.cls = take((size_t)kClsTables * (D.E + 1) * sizeof(int32_t));
    L.nb = (int)((M + kPlanChunk - 1) / kPlanChunk);
    L.hist = take((size_t)(L.nb > 0 ? L.nb : 1) * D.E * sizeof(int32_t));
    L.dwg_pieces = (long)(M / 64) + D.E;
    L.dwg_part = take((size_t)L.dwg_pieces * D.d * sizeof(float));
    L.dbg_part = take((size_t)L.dwg_pieces * sizeof(float));
    L.bias_part = take((size_t)L.dwg_pieces * (D.d > D.h ? D.d : D.h) * sizeof(float));
    L.gate_fail = take(((size_t)D.N + 1) * sizeof(int32_t));
    L.WgT = take((size_t)D.E * D.d * b);
    L.dense_chunks = (D.N + 511) / 512;
    if (D.score_all || D.balance_stats) {
        L.logits = take((size_t)D.N * D.E * sizeof(double));
        L.lse = take((size_t)D.N * sizeof(double));
        L.prob_part = take((size_t)(L.dense_chunks > 0 ? L.dense_chunks : 1) * D.E * sizeof(double));
    }
    if (D.score_all) {
        L.gate_S = take((size_t)D.N * sizeof(float));
        L.gate_R = take((size_t)D.N * D.E * sizeof(float));
        L.dx_dense = take((size_t)D.N * D.d * sizeof(float));
        L.dense_part = take((size_t)L.dense_chunks * D.E * D.d * sizeof(float));
        L.dense_bpart = take((size_t)L.dense_chunks * D.E * sizeof(float));
    }
    L.zeros = take(kZeroedBytes);
    L.sk_flags = L.zeros + kCtlFlags * sizeof(int32_t);
    L.sk_error = L.zeros + kCtlError * sizeof(int32_t);
    L.sk_part = take(D.dtype == MOE_BF16 ? (size_t)kSkPhases * kMaxPersistentWgs * kPartialBytesPerWg : 0);
    L.total = o;
    return L;
}

// ---- error reporting -------------------------------------------------------------------
void set_error(const char* fmt, ...);
// A launcher that could not launch (a function attribute was refused, no usable device): records the text and makes
// the next check_launch on this thread return MOE_ERR_HIP.
void fail_launch(const char* fmt, ...);
moe_status_t check_launch(const char* what);
constexpr int kMaxDevices = 64;   // per-device caches (function attributes, compute-unit counts) are indexed by the HIP device id
int current_device();             // the calling thread's HIP device, or -1 (after fail_launch)
moe_status_t check_desc(const moe_desc_t* D);   // host-side validation of a problem description (sets the error text)

// Kernels whose dynamic LDS exceeds the default limit: the kernel's limit is raised once per device (the static
// state is per kernel: one instance of this template each).  False after fail_launch.
template <typename Kern> static bool allow_dynamic_lds(Kern kern, int bytes)
{
    static std::mutex mu;
    static bool done[kMaxDevices] = {};
    const int dev = current_device();
    if (dev < 0) return false;
    std::lock_guard<std::mutex> lk(mu);
    if (!done[dev]) {
        const hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
        if (e != hipSuccess) { fail_launch("%d bytes of dynamic LDS refused on device %d: %s", bytes, dev, hipGetErrorString(e)); return false; }
        done[dev] = true;
    }
    return true;
}

// ---- kernel launchers (each enqueues on `st`; operand shapes are validated by the callers) ----
void launch_gate_topk(const moe_desc_t& D, const void* X, const void* Wg, const float* bg, int32_t* topk_idx,
                      float* topk_w, void* WgT, double* logits, double* lse, int32_t* gate_fail, hipStream_t st);
// bf16 with 17 to 256 experts and no caller of the stored logits: fp32 logits on the bf16 matrix cores with a certified
// margin, fp64 for the k selected logits and for the tokens that cannot be certified (gate_fail: [1 + N] int32 scratch)
void launch_gate_bf16(const moe_desc_t& D, const void* X, const void* Wg, const float* bg, int32_t* topk_idx, float* topk_w,
                      void* WgT, int32_t* gate_fail, hipStream_t st);
// (WgT: [E][d] scratch for the transposed gate matrix; logits [N][E] and lse [N]: only with desc.score_all, else NULL)
void launch_plan(const moe_desc_t& D, const WsLayout& L, const int32_t* topk_idx, int32_t* counts,
                 int32_t* offsets, int32_t* pos, int32_t* perm, char* ws, hipStream_t st);

void launch_scatter(const moe_desc_t& D, const void* X, const int32_t* perm, void* Xs, hipStream_t st);
void launch_combine(const moe_desc_t& D, const void* Ys, const float* topk_w, const int32_t* pos, void* Y,
                    hipStream_t st);
void launch_dcombine(const moe_desc_t& D, const void* dY, const void* Ys, const float* topk_w,
                     const int32_t* pos, void* dYs, float* dl, float* S_out, const void* X, void* Xs, hipStream_t st);
// (X, Xs: the scatter Xs[pos[a],:] = X[t,:] rides along, or NULL, NULL)
void launch_gate_bwd(const moe_desc_t& D, const WsLayout& L, const void* Xs, const void* dXs, const void* Wg,
                     const float* dl, const int32_t* topk_idx, const int32_t* pos, const int32_t* perm,
                     const int32_t* counts, const int32_t* offsets, void* dX, void* dWg, float* dbg, char* ws,
                     const void* X_dense, hipStream_t st);
void launch_balance_stats(const moe_desc_t& D, const WsLayout& L, const int32_t* counts, float* fraction, float* mean_prob,
                          float* loss, char* ws, hipStream_t st);
void launch_gate_dense(const moe_desc_t& D, const WsLayout& L, const void* X, const void* Wg, const int32_t* topk_idx,
                       char* ws, hipStream_t st);

// Grouped matrix products over the expert segments.
//   kRows*: C[r,:] (r in segment e) = A[r,:] * op(B[e]);  A is [M,K] row-major, C is [M,Nout] row-major.
//   kColsT: C[e] (K1 x K2) = A[seg e]^T * B[seg e];       A is [M,K1], B is [M,K2], C is [E,K1,K2].
enum GemmKind {
    kRowsNN_GeLU = 0,  // B[e] is [K,Nout];  writes C = acc (pre-activation) and C2 = GeLU(acc)
    kRowsNN = 1,       // B[e] is [K,Nout]
    kRowsNT_dGeLU = 2, // B[e] is [Nout,K];  C = acc * GeLU'(Zin)
    kRowsNT = 3,       // B[e] is [Nout,K]
    kColsT = 4         // weight gradient; honours grad_dtype and accumulate
};
struct GemmArgs {
    int kind;
    const void* A;
    const void* B;
    void* C;
    void* C2;         // kRowsNN_GeLU: GeLU output
    const void* Zin;  // kRowsNT_dGeLU: saved pre-activation [M,Nout]
    const void* bias; // kRowsNN_GeLU, kRowsNN: [E,Nout] added to the product (activation type), or NULL
    const int32_t* a_gather;  // kRows*: row r of the A operand is A[a_gather[r] / a_gather_div, :] (the scatter done on the fly), or NULL
    int a_gather_div;
    const int32_t* c_scatter; // kRowsNN: row r of the product is written to C[c_scatter[r], :] (the gather done on the fly; top-1 only), or NULL
    int K;            // kRows*: reduction width;  kColsT: K1 (rows of C[e])
    int Nout;         // kRows*: columns of C;     kColsT: K2 (columns of C[e])
    long M;           // total rows (N*k)
    int E;
    const int32_t* counts;
    const int32_t* offsets;
    const int32_t* tileP;  // [4][E+1]
    const int32_t* order;  // [E]
    const int32_t* cls;    // [kClsTables][E+1] size-class tables of the plan step, or NULL (bf16 row products only)
    const void* zeros;     // 1 KB of zeros
    void* sk_part;         // partial-sum tiles, one per phase and persistent workgroup
    int32_t* sk_flags;     // one flag per phase and persistent workgroup, all zero between launches
    int32_t* sk_error;
    const int32_t* by_expert;  // 1: the weight-gradient products give every XCD whole experts (decided by the plan step)
    long long* clock_probe;    // [2]: shader cycles and 100 MHz ticks of workgroup 0 of the last launch
    const int32_t* skewed;     // 1: the experts' sizes are strongly skewed (decided by the plan step)
    int32_t* dyn_counters;     // [9]: next tile of every XCD's list and the number of workgroups that have finished; zero between launches
    int whole_tiles;           // rows kinds: never cut a tile (another product in the same launch fills the idle workgroups)
    int on_demand;             // weight gradients: hand the tiles out from the counters whatever the sizes
    int stream_out;            // bf16 products: results leave as streaming stores (set by the host when the experts' weights exceed the L2 caches)
    int spin_limit;            // polls of a "partial sum ready" flag before the wait is given up and the status word set (negative: at once)
    int out_f32;      // kColsT: C holds float (else the activation type)
    int accumulate;   // kColsT
};
// Points the control-block fields of a GemmArgs at a workspace's control block.
inline void set_control(GemmArgs& a, char* ws, const WsLayout& L)
{
    int32_t* ctl = (int32_t*)(ws + L.zeros);
    a.zeros = ctl + kCtlZeroPage;
    a.sk_part = ws + L.sk_part;
    a.sk_flags = ctl + kCtlFlags;
    a.sk_error = ctl + kCtlError;
    a.by_expert = ctl + kCtlByExpert;
    a.clock_probe = (long long*)(ctl + kCtlClock);
    a.skewed = ctl + kCtlSkewed;
    a.dyn_counters = ctl + kCtlDyn;
}
void launch_segment_sums(const moe_desc_t& D, const WsLayout& L, const void* src, int width, const int32_t* counts,
                         const int32_t* offsets, float* out, char* ws, hipStream_t st);
void launch_ggemm_f32(const GemmArgs& a, hipStream_t st);
void launch_ggemm_bf16_sk(const GemmArgs& a, hipStream_t st);
// A rows kind (dZ or dXs) and a weight-gradient product that does not depend on it, in one launch.
void launch_ggemm_pair_bf16_sk(const GemmArgs& rows, const GemmArgs& cols, hipStream_t st);
bool ggemm_pair_pays(const GemmArgs& rows);   // whether the pair launch is expected to beat two launches

// ---- small device helpers ------------------------------------------------------------------
__device__ __forceinline__ float bf16_to_f32(unsigned short v) { return __uint_as_float(((unsigned)v) << 16); }
__device__ __forceinline__ unsigned short f32_to_bf16(float f)
{
    unsigned u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (unsigned short)((u >> 16) | 0x40);  // quiet NaN
    u += 0x7fffu + ((u >> 16) & 1u);                                                  // round to nearest even
    return (unsigned short)(u >> 16);
}
// Two floats -> two bf16 (round to nearest even) in one 32-bit word, low half = a: one v_cvt_pk_bf16_f32.
__device__ __forceinline__ unsigned pack_bf16x2(float a, float b)
{
    typedef __attribute__((ext_vector_type(2))) float f32x2_t;
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
    const f32x2_t v = {a, b};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2_t));
}
__device__ __forceinline__ float gelu_f(float z) { return 0.5f * z * (1.0f + erff(z * 0.70710678118654752f)); }
__device__ __forceinline__ float gelu_grad_f(float z)
{
    return 0.5f * (1.0f + erff(z * 0.70710678118654752f)) + z * __expf(-0.5f * z * z) * 0.39894228040143268f;
}


}  // namespace moe
