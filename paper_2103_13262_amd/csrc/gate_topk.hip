// Gate score, top-k selection and combine weights (Algorithm 1: "score <- G(x)",
// "indices <- ArgMax_k(score)"; the gate is one fully-connected layer, Section 5.2).
//
// A group of SG lanes (a power of two, SG <= 64) of one wavefront owns one token; lane sl of
// the group owns experts sl, sl+SG, ...  (the gate matrix is shared through LDS)  Logits are accumulated in fp64 in ascending feature
// order starting from the bias: the products of two fp32-representable numbers are exact in
// fp64, so the selection is that of exact arithmetic (ties -> lower expert id) up to fp64
// summation rounding (~1e-16 relative; equal columns of the gate matrix still give equal logits).  Selection is k rounds of a butterfly arg-max over the group.
#include <cstdlib>
#include <type_traits>

#include "common.h"

namespace moe {

template <typename T> struct Elem;
template <> struct Elem<float> {
    static __device__ __forceinline__ double get(const float* p, size_t i) { return (double)p[i]; }
};
template <> struct Elem<unsigned short> {
    static __device__ __forceinline__ double get(const unsigned short* p, size_t i) { return (double)bf16_to_f32(p[i]); }
};

// One workgroup = 4 wavefronts; every wavefront handles TPW token groups of G = 64/SG tokens.  The gate
// matrix is staged through LDS in slabs of DC feature rows (all tokens of the workgroup share it), the
// token rows are read 8 features at a time.  Per (token, expert) the sum runs in ascending feature order.
template <typename T, int R, int TPW>
__global__ __launch_bounds__(256) void gate_topk_kernel(const T* __restrict__ X, const T* __restrict__ Wg,
                                                        const float* __restrict__ bg, int N, int d, int E, int k,
                                                        int SG, int DC, int32_t* __restrict__ topk_idx,
                                                        float* __restrict__ topk_w)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    T* sW = reinterpret_cast<T*>(smem_raw);          // [DC][E]   slab of the gate matrix
    T* sX = sW + (size_t)DC * E;                     // [TB][DC]  the same feature slab of this workgroup's tokens
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int G = 64 / SG;
    const int TB = 4 * G * TPW;                      // tokens per workgroup
    const long tok0 = (long)blockIdx.x * TB;
    const int sl = lane & (SG - 1), g = lane / SG;
    const double ninf = -__builtin_inf();
    int tl[TPW];                                     // token of group q, local to the workgroup
    // NCH independent partial sums per logit (feature i goes to chain i % NCH) hide the latency of the
    // dependent fp64 FMA chain; they are combined pairwise at the end and the bias is added last.
    constexpr int NCH = (R * TPW >= 8) ? 1 : (R * TPW >= 4) ? 2 : 4;
    double part[TPW][R][NCH];
#pragma unroll
    for (int q = 0; q < TPW; ++q) {
        tl[q] = q * (4 * G) + wave * G + g;
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int c = 0; c < NCH; ++c) part[q][r][c] = 0.0;
    }
    int ecl[R];   // own experts, clamped: lanes past E compute a copy that is discarded (keeps the loop branch-free)
#pragma unroll
    for (int r = 0; r < R; ++r) ecl[r] = min(r * SG + sl, E - 1);
    constexpr int V = 16 / sizeof(T);                // elements per 16-byte piece
    for (int c0 = 0; c0 < d; c0 += DC) {
        const int rows = min(DC, d - c0);
        __syncthreads();   // previous slab fully consumed
        {
            const uint4* src = reinterpret_cast<const uint4*>(Wg + (size_t)c0 * E);
            uint4* dst = reinterpret_cast<uint4*>(sW);
            const int n16 = (int)((size_t)rows * E / V);
            for (int i = threadIdx.x; i < n16; i += 256) dst[i] = src[i];
            const int cpr = rows / V;                // 16-byte pieces per token row of the slab
            for (int i = threadIdx.x; i < TB * cpr; i += 256) {
                const int tt = i / cpr, c = i - tt * cpr;
                const long t = tok0 + tt < N ? tok0 + tt : (long)N - 1;
                reinterpret_cast<uint4*>(sX + (size_t)tt * DC)[c] =
                    reinterpret_cast<const uint4*>(X + (size_t)t * d + c0)[c];
            }
        }
        __syncthreads();
#pragma unroll
        for (int q = 0; q < TPW; ++q) {
            const T* xr = sX + (size_t)tl[q] * DC;
            for (int i = 0; i < rows; i += 8) {
                double x[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) x[u] = Elem<T>::get(xr, i + u);
#pragma unroll
                for (int u = 0; u < 8; ++u) {
#pragma unroll
                    for (int r = 0; r < R; ++r)
                        part[q][r][u % NCH] =
                            fma(x[u], Elem<T>::get(sW, (size_t)(i + u) * E + ecl[r]), part[q][r][u % NCH]);
                }
            }
        }
    }
    double acc[TPW][R];
#pragma unroll
    for (int q = 0; q < TPW; ++q)
#pragma unroll
        for (int r = 0; r < R; ++r) {
            double s = part[q][r][0];
            if constexpr (NCH == 2) s = part[q][r][0] + part[q][r][1];
            if constexpr (NCH == 4) s = (part[q][r][0] + part[q][r][1]) + (part[q][r][2] + part[q][r][3]);
            const int e = r * SG + sl;
            acc[q][r] = s + ((bg && e < E) ? (double)bg[e] : 0.0);
        }
#pragma unroll
    for (int q = 0; q < TPW; ++q) {
        const long t = tok0 + tl[q];
        const bool tv = t < N;
#pragma unroll
        for (int r = 0; r < R; ++r)   // NaN ranks last and experts past E never win: indices stay in range
            if (!(acc[q][r] == acc[q][r]) || r * SG + sl >= E) acc[q][r] = ninf;

        unsigned taken = 0;
        double sel[kMaxK];
        int seli[kMaxK];
#pragma unroll
        for (int j = 0; j < kMaxK; ++j) {
            if (j < k) {
                double bv = ninf;
                int be = 0x7fffffff;
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    const int e = r * SG + sl;
                    if (e < E && !((taken >> r) & 1u) && (acc[q][r] > bv || (acc[q][r] == bv && e < be))) {
                        bv = acc[q][r];
                        be = e;
                    }
                }
                for (int off = SG >> 1; off > 0; off >>= 1) {
                    const double ov = __shfl_xor(bv, off, 64);
                    const int oe = __shfl_xor(be, off, 64);
                    if (ov > bv || (ov == bv && oe < be)) {
                        bv = ov;
                        be = oe;
                    }
                }
                sel[j] = bv;
                seli[j] = be;
                if ((be & (SG - 1)) == sl) taken |= 1u << (be / SG);
            }
        }
        if (tv && sl == 0) {
            double ex[kMaxK], den = 0.0;
#pragma unroll
            for (int j = 0; j < kMaxK; ++j)
                if (j < k) {
                    ex[j] = exp(sel[j] - sel[0]);
                    den += ex[j];
                }
#pragma unroll
            for (int j = 0; j < kMaxK; ++j)
                if (j < k) {
                    topk_idx[t * k + j] = seli[j];
                    topk_w[t * k + j] = (float)(ex[j] / den);
                }
        }
    }
}

template <typename T>
static void launch_typed(const moe_desc_t& D, const T* X, const T* Wg, const float* bg, int32_t* idx, float* w,
                         hipStream_t st)
{
    int SG = 1;
    while (SG < D.E && SG < 64) SG <<= 1;
    const int R = (D.E + SG - 1) / SG;  // 1..16
    const int G = 64 / SG;
    const long per_tpw = 4L * G;
    // several token groups per wavefront only when that still leaves enough workgroups to fill the chip
    const int tpw = (R <= 2 && (D.N + per_tpw * 4 - 1) / (per_tpw * 4) >= 1024) ? 4
                  : (R <= 4 && (D.N + per_tpw * 2 - 1) / (per_tpw * 2) >= 1024) ? 2 : 1;
    const int TB = (int)per_tpw * tpw;
    constexpr int kSlabBytes = 65536;    // gate slab [DC][E] plus token slab [TB][DC]
    int DC = (int)(kSlabBytes / ((size_t)(D.E + TB) * sizeof(T))) / 8 * 8;
    if (DC < 8) DC = 8;
    if (DC > D.d) DC = D.d;
    const size_t lds = (size_t)DC * (D.E + TB) * sizeof(T);
    const unsigned grid = (unsigned)((D.N + TB - 1) / TB);
    auto go = [&](auto rr, auto tt) {
        constexpr int RR = decltype(rr)::value, TT = decltype(tt)::value;
        auto kern = gate_topk_kernel<T, RR, TT>;
        if (lds > 48 * 1024 &&
            hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
            return;   // launch skipped; the caller's hipGetLastError() reports the failure
        hipLaunchKernelGGL(kern, dim3(grid), dim3(256), lds, st, X, Wg, bg, D.N, D.d, D.E, D.k, SG, DC, idx, w);
    };
    using std::integral_constant;
#define IC(v) integral_constant<int, v>{}
    if (tpw == 4) go(IC(1), IC(4)); else if (tpw == 2) go(IC(1), IC(2)); else go(IC(1), IC(1));   // E <= 16: R = 1
#undef IC
}

// Sorted list of the k best (value, expert) pairs of one token, kept in registers.
__device__ __forceinline__ void topk_insert(double cv, int ce, double (&v)[kMaxK], int (&id)[kMaxK], int k)
{   // keeps v descending, equal values by ascending expert id
#pragma unroll
    for (int j = 0; j < kMaxK; ++j) {
        if (j < k && (cv > v[j] || (cv == v[j] && ce < id[j]))) {
            const double tv = v[j]; v[j] = cv; cv = tv;
            const int ti = id[j]; id[j] = ce; ce = ti;
        }
    }
}

// ---- matrix-core variant: logits as an fp64 product on v_mfma_f64_16x16x4_f64 -------------------------
// Workgroup = 64 tokens (16 per wavefront) x blocks of 64 experts.  Token features and gate columns are widened
// to fp64 while they are staged into LDS (feature-major, 32 features per slab); every 4-deep step is one LDS
// read for the token operand and one per 16 experts for the gate operand.  Operand lane l holds row/column
// l%16 at depth l/16; result register r of lane l is token 4r + l/16, expert l%16.  The logits of a block are
// passed through LDS and scanned token-per-lane (16 experts per wavefront) into sorted k-lists.
typedef __attribute__((ext_vector_type(4))) double f64x4;

template <typename T, int NT>
__global__ __launch_bounds__(256) void gate_mfma_kernel(const T* __restrict__ X, const T* __restrict__ Wg,
                                                        const float* __restrict__ bg, int N, int d, int E, int k,
                                                        int32_t* __restrict__ topk_idx, float* __restrict__ topk_w)
{
    constexpr int KC = 32, V = 16 / sizeof(T), NPX = 8 / V;   // features per slab; 16-byte pieces per thread
    constexpr int EB = 16 * NT;                               // experts per block (NT groups of 16)
    __shared__ __align__(16) double smem[2 * KC * 64];      // sX [KC][64 tokens] | sW [KC][64 experts]; reused
    double* sX = smem;
    double* sW = smem + KC * 64;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const long tok0 = (long)blockIdx.x * 64;
    const double ninf = -__builtin_inf();
    // staging roles: token features -> thread (token = tid % 64, 8-feature group = tid / 64)
    const long trow = tok0 + lane < N ? tok0 + lane : (long)N - 1;
    const T* xsrc = X + (size_t)trow * d + wave * 8;
    // gate slab -> thread (feature = tid / 8, 8 experts from (tid % 8) * 8)
    const int wf = threadIdx.x >> 3, we = (threadIdx.x & 7) * 8;

    double v[kMaxK];
    int id[kMaxK];
#pragma unroll
    for (int j = 0; j < kMaxK; ++j) { v[j] = ninf; id[j] = 0x7fffffff; }

    for (int eb0 = 0; eb0 < E; eb0 += EB) {
        f64x4 acc[NT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[nt] = f64x4{0.0, 0.0, 0.0, 0.0};

        uint4 pre[NPX];
#pragma unroll
        for (int q = 0; q < NPX; ++q) pre[q] = reinterpret_cast<const uint4*>(xsrc)[q];
        for (int c0 = 0; c0 < d; c0 += KC) {
            __syncthreads();                                 // previous slab (or the logit patch) fully consumed
            {
                T tmp[8];
#pragma unroll
                for (int q = 0; q < NPX; ++q) reinterpret_cast<uint4*>(tmp)[q] = pre[q];
#pragma unroll
                for (int u = 0; u < 8; ++u) sX[(wave * 8 + u) * 64 + lane] = Elem<T>::get(tmp, u);
                const T* wrow = Wg + (size_t)(c0 + wf) * E + eb0 + we;
                if (we < EB) {
#pragma unroll
                    for (int u = 0; u < 8; ++u)
                        sW[wf * 64 + we + u] = eb0 + we + u < E ? Elem<T>::get(wrow, u) : 0.0;
                }
            }
            if (c0 + KC < d) {
#pragma unroll
                for (int q = 0; q < NPX; ++q) pre[q] = reinterpret_cast<const uint4*>(xsrc + c0 + KC)[q];
            }
            __syncthreads();
#pragma unroll
            for (int kk = 0; kk < KC / 4; ++kk) {
                const int row = (kk * 4 + (lane >> 4)) * 64 + (lane & 15);
                const double a = sX[row + wave * 16];
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    acc[nt] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, sW[row + nt * 16], acc[nt], 0, 0, 0);
            }
        }
        __syncthreads();                                     // all waves are done with the slabs
        double* sL = smem;                                   // [64 tokens][64 experts]
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int r = 0; r < 4; ++r)
                sL[(wave * 16 + 4 * r + (lane >> 4)) * 64 + nt * 16 + (lane & 15)] = acc[nt][r];
        __syncthreads();
        for (int e = 0; e < EB / 4; ++e) {                   // lane = token, this wavefront's quarter of the block
            const int ge = eb0 + wave * (EB / 4) + e;
            if (ge < E) {                                    // wave-uniform
                double l = sL[lane * 64 + wave * (EB / 4) + e] + (bg ? (double)bg[ge] : 0.0);
                if (!(l == l)) l = ninf;                     // NaN ranks last; indices stay in range
                topk_insert(l, ge, v, id, k);
            }
        }
    }
    // merge the four per-wavefront lists
    __syncthreads();
    double* mV = smem;                                       // [wave][slot][token]
    int* mI = reinterpret_cast<int*>(smem + 4 * kMaxK * 64);
#pragma unroll
    for (int j = 0; j < kMaxK; ++j)
        if (j < k) {
            mV[(wave * kMaxK + j) * 64 + lane] = v[j];
            mI[(wave * kMaxK + j) * 64 + lane] = id[j];
        }
    __syncthreads();
    if (wave == 0) {
        for (int w = 1; w < 4; ++w)
#pragma unroll
            for (int j = 0; j < kMaxK; ++j)
                if (j < k) topk_insert(mV[(w * kMaxK + j) * 64 + lane], mI[(w * kMaxK + j) * 64 + lane], v, id, k);
        const long t = tok0 + lane;
        if (t < N) {
            double ex[kMaxK], den = 0.0;
#pragma unroll
            for (int j = 0; j < kMaxK; ++j)
                if (j < k) {
                    ex[j] = exp(v[j] - v[0]);
                    den += ex[j];
                }
#pragma unroll
            for (int j = 0; j < kMaxK; ++j)
                if (j < k) {
                    topk_idx[t * k + j] = id[j];
                    topk_w[t * k + j] = (float)(ex[j] / den);
                }
        }
    }
}

template <typename T>
static void launch_mfma(const moe_desc_t& D, const T* X, const T* Wg, const float* bg, int32_t* idx, float* w, hipStream_t st)
{
    const dim3 grid((unsigned)((D.N + 63) / 64));
    if (D.E <= 32)
        hipLaunchKernelGGL((gate_mfma_kernel<T, 2>), grid, dim3(256), 0, st, X, Wg, bg, D.N, D.d, D.E, D.k, idx, w);
    else
        hipLaunchKernelGGL((gate_mfma_kernel<T, 4>), grid, dim3(256), 0, st, X, Wg, bg, D.N, D.d, D.E, D.k, idx, w);
}

void launch_gate_topk(const moe_desc_t& D, const void* X, const void* Wg, const float* bg, int32_t* topk_idx,
                      float* topk_w, hipStream_t st)
{
    // Few experts: a group of lanes per token with the products on the vector ALU wastes nothing; from 17 experts
    // on the fp64 matrix cores win (measured: E=16 33 vs 79 us, E=32 527 vs 231 us, E=256 610 vs 157 us).
    const bool lanes_over_experts = D.E <= 16;
    if (D.dtype == MOE_BF16) {
        using T = unsigned short;
        if (lanes_over_experts) launch_typed<T>(D, (const T*)X, (const T*)Wg, bg, topk_idx, topk_w, st);
        else launch_mfma<T>(D, (const T*)X, (const T*)Wg, bg, topk_idx, topk_w, st);
    } else {
        using T = float;
        if (lanes_over_experts) launch_typed<T>(D, (const T*)X, (const T*)Wg, bg, topk_idx, topk_w, st);
        else launch_mfma<T>(D, (const T*)X, (const T*)Wg, bg, topk_idx, topk_w, st);
    }
}

}  // namespace moe
