// Gate score, top-k selection and combine weights (Algorithm 1: "score <- G(x)",
// "indices <- ArgMax_k(score)"; the gate is one fully-connected layer, Section 5.2).
//
// A group of SG lanes (a power of two, SG <= 64) of one wavefront owns one token; lane sl of
// the group owns experts sl, sl+SG, ...  Logits are accumulated in fp64 in ascending feature
// order starting from the bias: the products of two fp32-representable numbers are exact in
// fp64, so the selection is that of exact arithmetic (ties -> lower expert id) up to fp64
// summation rounding.  Selection is k rounds of a butterfly arg-max over the group.
#include "common.h"

namespace moe {

template <typename T> struct Elem;
template <> struct Elem<float> {
    static __device__ __forceinline__ double get(const float* p, size_t i) { return (double)p[i]; }
};
template <> struct Elem<unsigned short> {
    static __device__ __forceinline__ double get(const unsigned short* p, size_t i) { return (double)bf16_to_f32(p[i]); }
};

template <typename T, int R>
__global__ __launch_bounds__(256) void gate_topk_kernel(const T* __restrict__ X, const T* __restrict__ Wg,
                                                        const float* __restrict__ bg, int N, int d, int E, int k,
                                                        int SG, int32_t* __restrict__ topk_idx,
                                                        float* __restrict__ topk_w)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int G = 64 / SG;
    const int sl = lane & (SG - 1), g = lane / SG;
    const long t = ((long)blockIdx.x * 4 + wave) * G + g;
    const bool tv = t < N;
    const size_t trow = (size_t)(tv ? t : (N - 1)) * d;
    const double ninf = -__builtin_inf();

    double acc[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int e = r * SG + sl;
        acc[r] = e < E ? (bg ? (double)bg[e] : 0.0) : ninf;
    }
    for (int i = 0; i < d; i += 8) {
        double x[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) x[u] = Elem<T>::get(X, trow + i + u);
#pragma unroll
        for (int u = 0; u < 8; ++u) {
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const int e = r * SG + sl;
                if (e < E) acc[r] = fma(x[u], Elem<T>::get(Wg, (size_t)(i + u) * E + e), acc[r]);
            }
        }
    }
#pragma unroll
    for (int r = 0; r < R; ++r)
        if (!(acc[r] == acc[r])) acc[r] = ninf;  // NaN ranks last; indices stay in range

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
                if (e < E && !((taken >> r) & 1u) && (acc[r] > bv || (acc[r] == bv && e < be))) {
                    bv = acc[r];
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

template <typename T>
static void launch_typed(const moe_desc_t& D, const T* X, const T* Wg, const float* bg, int32_t* idx, float* w,
                         hipStream_t st)
{
    int SG = 1;
    while (SG < D.E && SG < 64) SG <<= 1;
    const int R = (D.E + SG - 1) / SG;  // 1..16
    const int G = 64 / SG;
    const unsigned grid = (unsigned)((D.N + 4 * G - 1) / (4 * G));
#define MOE_GATE(RR)                                                                                         \
    hipLaunchKernelGGL((gate_topk_kernel<T, RR>), dim3(grid), dim3(256), 0, st, X, Wg, bg, D.N, D.d, D.E, D.k, \
                       SG, idx, w)
    if (R <= 1) MOE_GATE(1);
    else if (R <= 2) MOE_GATE(2);
    else if (R <= 4) MOE_GATE(4);
    else if (R <= 8) MOE_GATE(8);
    else MOE_GATE(16);
#undef MOE_GATE
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
