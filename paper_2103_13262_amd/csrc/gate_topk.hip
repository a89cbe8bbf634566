// Gate score, top-k selection and combine weights (Algorithm 1: "score <- G(x)",
// "indices <- ArgMax_k(score)"; the gate is one fully-connected layer, Section 5.2).
//
// A group of SG lanes (a power of two, SG <= 64) of one wavefront owns one token; lane sl of
// the group owns experts sl, sl+SG, ...  (the gate matrix is shared through LDS)  Logits are accumulated in fp64 in ascending feature
// order starting from the bias: the products of two fp32-representable numbers are exact in
// fp64, so the selection is that of exact arithmetic (ties -> lower expert id) up to fp64
// summation rounding (~1e-16 relative; equal columns of the gate matrix still give equal logits).  Selection is k rounds of a butterfly arg-max over the group.
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
    if (R <= 1) { if (tpw == 4) go(IC(1), IC(4)); else if (tpw == 2) go(IC(1), IC(2)); else go(IC(1), IC(1)); }
    else if (R <= 2) { if (tpw == 4) go(IC(2), IC(4)); else if (tpw == 2) go(IC(2), IC(2)); else go(IC(2), IC(1)); }
    else if (R <= 4) { if (tpw == 2) go(IC(4), IC(2)); else go(IC(4), IC(1)); }
    else if (R <= 8) go(IC(8), IC(1));
    else go(IC(16), IC(1));
#undef IC
}

void launch_gate_topk(const moe_desc_t& D, const void* X, const void* Wg, const float* bg, int32_t* topk_idx,
                      float* topk_w, hipStream_t st)
{
    if (D.dtype == MOE_BF16)
        launch_typed<unsigned short>(D, (const unsigned short*)X, (const unsigned short*)Wg, bg, topk_idx, topk_w, st);
    else
        launch_typed<float>(D, (const float*)X, (const float*)Wg, bg, topk_idx, topk_w, st);
}

}  // namespace moe
