// Gate score, top-k selection and combine weights (Algorithm 1: "score <- G(x)",
// "indices <- ArgMax_k(score)"; the gate is one fully-connected layer, Section 5.2).
//
// The logits are an fp64 product on the matrix cores (v_mfma_f64_16x16x4_f64), accumulated from zero in a fixed
// order with the bias added last: the products of two fp32-representable numbers are exact in fp64, so the
// selection is that of exact arithmetic (ties -> lower expert id) up to fp64 summation rounding (~1e-16
// relative; equal columns of the gate matrix still give equal logits).  Operand lane l holds row / column l%16
// at depth l/16; result register r of lane l is token 4r + l/16, expert l%16.  Up to 16 experts: one workgroup
// per 16 tokens with the reduction split over its four wavefronts; up to 32: 64 tokens per workgroup, a wavefront
// per 16 tokens; more: blocks of 64 experts, a wavefront per 16 experts.
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

// Feature j (0..7, a compile-time constant where it is used) of 8 consecutive features held in registers as
// 16-byte pieces, widened to fp64.  (Kept as pieces and taken apart with shifts: an element array filled through
// a pointer cast ends up in scratch memory.)
template <typename T> struct Piece;
template <> struct Piece<unsigned short> {
    static constexpr int N = 1;
    static __device__ __forceinline__ double get(const uint4 (&p)[1], int j)
    {
        const unsigned w = j < 2 ? p[0].x : j < 4 ? p[0].y : j < 6 ? p[0].z : p[0].w;
        return (double)__uint_as_float((j & 1) ? (w & 0xffff0000u) : (w << 16));
    }
};
template <> struct Piece<float> {
    static constexpr int N = 2;
    static __device__ __forceinline__ double get(const uint4 (&p)[2], int j)
    {
        const uint4& q = p[j >> 2];
        const unsigned w = (j & 3) == 0 ? q.x : (j & 3) == 1 ? q.y : (j & 3) == 2 ? q.z : q.w;
        return (double)__uint_as_float(w);
    }
};

// A 16-byte piece as a value.  (Copying an element of a register array straight to LDS is compiled as a memory
// copy, which keeps the whole array in scratch memory - and puts the wait for a prefetch right behind the load.)
__device__ __forceinline__ uint4 by_value(const uint4& p) { return make_uint4(p.x, p.y, p.z, p.w); }

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

typedef __attribute__((ext_vector_type(4))) double f64x4;

// ---- up to 16 experts -----------------------------------------------------------------------------------
// Workgroup = 16 tokens x 16 expert columns (columns past E are zero).  The token rows and the transposed gate
// matrix are staged in LDS in their storage type, a slab of 256 features at a time; lane l reads 8 consecutive
// features of token / expert l%16 at offset 8*(l/16) of a 32-feature group and widens them to fp64 on the way
// into eight matrix-core steps (even and odd steps feed two accumulators, added at the end).  Wavefront w takes
// the 32-feature groups w, w+4, ...; the four partial sums of a logit are added in the order ((0 + 1) + 2) + 3.
template <typename T>
__global__ __launch_bounds__(256) void gate_mfma16_kernel(const T* __restrict__ X, const T* __restrict__ Wg,
                                                          const float* __restrict__ bg, int N, int d, int E, int k,
                                                          int32_t* __restrict__ topk_idx, float* __restrict__ topk_w,
                                                          double* __restrict__ logits_out)
{
    constexpr int V = 16 / sizeof(T);                // elements per 16-byte piece
    constexpr int DC = 256;                          // features per slab
    constexpr int PP = DC / (16 * V);                // 16-byte pieces per thread and slab, of either operand
    constexpr int S = DC + V;                        // row stride: consecutive rows start 16 bytes apart in the banks
    constexpr int kSlabBytes = 2 * 16 * S * (int)sizeof(T), kTailBytes = 5 * 256 * (int)sizeof(double);
    __shared__ __align__(16) unsigned char smem_raw[kSlabBytes > kTailBytes ? kSlabBytes : kTailBytes];
    T* sX = reinterpret_cast<T*>(smem_raw);          // [16 tokens][S]
    T* sW = sX + 16 * S;                             // [16 experts][S]  (transposed slab of the gate matrix)
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const long tok0 = (long)blockIdx.x * 16;
    // The next slab travels from memory into registers while the matrix cores work on the current one.
    uint4 px[PP], pw[PP];
    auto fetch = [&](int c0) {
        // (every thread loads every time, indices past the end clamped)
        const int rows = min(DC, d - c0), cpr = rows / V, n16 = rows * E / V;
        const T* wsrc = Wg + (size_t)c0 * E;         // the gate slab [rows][E] is contiguous in memory
#pragma unroll
        for (int u = 0; u < PP; ++u) {
            const int i = threadIdx.x + u * 256;
            const int ix = min(i, 16 * cpr - 1);
            const int tt = ix / cpr, c = ix - tt * cpr;
            const long t = tok0 + tt < N ? tok0 + tt : (long)N - 1;
            px[u] = reinterpret_cast<const uint4*>(X + (size_t)t * d + c0)[c];
            pw[u] = reinterpret_cast<const uint4*>(wsrc)[min(i, n16 - 1)];
        }
    };
    auto stash = [&](int c0) {
        const int rows = min(DC, d - c0), cpr = rows / V, n16 = rows * E / V;
#pragma unroll
        for (int u = 0; u < PP; ++u) {
            const int i = threadIdx.x + u * 256;
            if (i < 16 * cpr) {
                const int tt = i / cpr, c = i - tt * cpr;
                *reinterpret_cast<uint4*>(sX + tt * S + c * V) = by_value(px[u]);
            }
            if (i < n16) {                           // element (f, e) of the slab goes to sW[e][f]
                const T* el = reinterpret_cast<const T*>(&pw[u]);
                int f = i * V / E, e = i * V - f * E;
#pragma unroll
                for (int q = 0; q < V; ++q) {
                    sW[e * S + f] = el[q];
                    if (++e == E) { e = 0; ++f; }
                }
            }
        }
    };
    if (E < 16)                                      // columns past E: zeros, written once
        for (int i = threadIdx.x; i < (16 - E) * S; i += 256) sW[E * S + i] = T(0);
    f64x4 acc = f64x4{0.0, 0.0, 0.0, 0.0}, acc2 = acc;
    const T* xa = sX + (lane & 15) * S + (lane >> 4) * 8;
    const T* wb = sW + (lane & 15) * S + (lane >> 4) * 8;
    fetch(0);
    for (int c0 = 0; c0 < d; c0 += DC) {
        const int rows = min(DC, d - c0);            // a multiple of 32
        __syncthreads();                             // previous slab fully consumed
        stash(c0);
        __syncthreads();
        if (c0 + DC < d) fetch(c0 + DC);
        for (int grp = wave; grp < rows / 32; grp += 4) {
            uint4 xt[Piece<T>::N], wt[Piece<T>::N];
#pragma unroll
            for (int q = 0; q < Piece<T>::N; ++q) {
                xt[q] = reinterpret_cast<const uint4*>(xa + grp * 32)[q];
                wt[q] = reinterpret_cast<const uint4*>(wb + grp * 32)[q];
            }
#pragma unroll
            for (int j = 0; j < 8; j += 2) {         // two independent chains: a step does not wait for the one before
                acc = __builtin_amdgcn_mfma_f64_16x16x4f64(Piece<T>::get(xt, j), Piece<T>::get(wt, j), acc, 0, 0, 0);
                acc2 = __builtin_amdgcn_mfma_f64_16x16x4f64(Piece<T>::get(xt, j + 1), Piece<T>::get(wt, j + 1), acc2, 0, 0, 0);
            }
        }
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) acc[r] += acc2[r];
    __syncthreads();                                 // all waves are done with the slabs
    double* sP = reinterpret_cast<double*>(smem_raw);   // [4 waves][16 tokens][16 experts]
    double* sL = sP + 4 * 256;                          // [16 tokens][16 experts]
#pragma unroll
    for (int r = 0; r < 4; ++r) sP[wave * 256 + (4 * r + (lane >> 4)) * 16 + (lane & 15)] = acc[r];
    __syncthreads();
    {
        const int i = threadIdx.x, e = i & 15;
        double l = ((sP[i] + sP[256 + i]) + sP[512 + i]) + sP[768 + i];
        if (bg && e < E) l += (double)bg[e];
        if (!(l == l) || e >= E) l = -__builtin_inf();   // NaN ranks last; columns past E never win
        sL[i] = l;
        if (logits_out && e < E && tok0 + (i >> 4) < N) logits_out[(size_t)(tok0 + (i >> 4)) * E + e] = l;
    }
    __syncthreads();
    {
        // Selection by rank, one thread per (token, expert): the rank of a logit is the number of logits of the same
        // token that beat it (larger, or equal with a lower expert id); ranks below k are the slots.
        const int i = threadIdx.x, tt = i >> 4, e = i & 15;
        const double mine = sL[i];
        int rank = 0;
#pragma unroll
        for (int o = 0; o < 16; ++o) {
            const double other = sL[tt * 16 + o];
            rank += (o < E && (other > mine || (other == mine && o < e))) ? 1 : 0;
        }
        double* sSel = sP;                           // [16 tokens][kMaxK] selected logits by slot (the partial sums are dead)
        int* sIdx = reinterpret_cast<int*>(sP + 16 * kMaxK);
        __syncthreads();
        if (e < E && rank < k) { sSel[tt * kMaxK + rank] = mine; sIdx[tt * kMaxK + rank] = e; }
        __syncthreads();
        const long t = tok0 + tt;
        if (e < k && t < N) {                        // thread (token, slot)
            const double top = sSel[tt * kMaxK];
            double den = 0.0;
            for (int j = 0; j < k; ++j) den += exp(sSel[tt * kMaxK + j] - top);
            topk_idx[t * k + e] = sIdx[tt * kMaxK + e];
            topk_w[t * k + e] = (float)(exp(sSel[tt * kMaxK + e] - top) / den);
        }
    }
}

template <typename T>
static void launch_mfma16(const moe_desc_t& D, const T* X, const T* Wg, const float* bg, int32_t* idx, float* w,
                          double* logits, hipStream_t st)
{
    hipLaunchKernelGGL(gate_mfma16_kernel<T>, dim3((unsigned)((D.N + 15) / 16)), dim3(256), 0, st, X, Wg, bg, D.N, D.d, D.E,
                       D.k, idx, w, logits);
}

// ---- 17 to 32 experts -----------------------------------------------------------------------------------------
// Workgroup = 64 tokens (16 per wavefront) x blocks of 32 experts.  Token features and gate columns are widened
// to fp64 while they are staged into LDS (feature-major, 32 features per slab); every 4-deep step is one LDS
// read for the token operand and one per 16 experts for the gate operand.  Operand lane l holds row/column
// l%16 at depth l/16; result register r of lane l is token 4r + l/16, expert l%16.  The logits of a block are
// passed through LDS and scanned token-per-lane (16 experts per wavefront) into sorted k-lists.
template <typename T, int NT>
__global__ __launch_bounds__(256) void gate_mfma_kernel(const T* __restrict__ X, const T* __restrict__ Wg,
                                                        const float* __restrict__ bg, int N, int d, int E, int k,
                                                        int32_t* __restrict__ topk_idx, float* __restrict__ topk_w,
                                                        double* __restrict__ logits_out)
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
                if (logits_out && tok0 + lane < N) logits_out[(size_t)(tok0 + lane) * E + ge] = l;
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

// ---- more than 32 experts -----------------------------------------------------------------------------------
// Workgroup = 16*MT tokens x blocks of 64 experts; wavefront w owns the 16 experts w of the block for all the
// tokens, so a gate operand register feeds MT matrix-core steps.  Both operands are staged in LDS in their storage
// type, 512 bytes of every row per slab (the gate matrix is read from its transpose, written by a small kernel
// before this one, so that an expert's features are contiguous); lane l reads 8 consecutive features of token /
// expert l%16 at offset 8*(l/16) of a 32-feature group and widens them to fp64 on the way into eight steps.  The
// next slab travels from memory into registers meanwhile.  A logit is one accumulator chain over the features in
// ascending (slab, group, step) order, the same for every expert.  Selection as in the kernel above.
template <typename T>
__global__ __launch_bounds__(256) void gate_transpose(const T* __restrict__ Wg, T* __restrict__ WgT, int d, int E)
{
    const long i = (long)blockIdx.x * 256 + threadIdx.x;   // index into WgT [E][d]
    if (i < (long)d * E) {
        const int e = (int)(i / d), f = (int)(i - (long)e * d);
        WgT[i] = Wg[(size_t)f * E + e];
    }
}

template <typename T, int MT>
__global__ __launch_bounds__(256) void gate_mfma_wide_kernel(const T* __restrict__ X, const T* __restrict__ WgT,
                                                             const float* __restrict__ bg, int N, int d, int E, int k,
                                                             int32_t* __restrict__ topk_idx, float* __restrict__ topk_w,
                                                             double* __restrict__ logits_out)
{
    constexpr int V = 16 / sizeof(T);                // elements per 16-byte piece
    constexpr int DC = 512 / sizeof(T);              // features per slab
    constexpr int CPR = 32;                          // 16-byte pieces per row and slab
    constexpr int S = DC + V;                        // row stride: consecutive rows start 16 bytes apart in the banks
    constexpr int TT = 16 * MT;                      // tokens per workgroup
    constexpr int PX = TT * CPR / 256, PW = 64 * CPR / 256;
    constexpr int CH = MT == 1 ? 2 : 1;              // accumulator chains per token group
    extern __shared__ __align__(16) unsigned char smem_raw[];
    T* sX = reinterpret_cast<T*>(smem_raw);          // [TT tokens][S]
    T* sW = sX + TT * S;                             // [64 experts][S]
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const long tok0 = (long)blockIdx.x * TT;
    const double ninf = -__builtin_inf();
    const int nslab = (d + DC - 1) / DC, nblk = (E + 63) / 64;

    uint4 px[PX], pw[PW];
    auto fetch = [&](int eb0, int c0) {
        // (every thread loads every time; pieces past the end of a short last slab repeat its last piece and are
        // not stored)
        const int cpr = min(DC, d - c0) / V;
        const int c = min((int)threadIdx.x & (CPR - 1), cpr - 1), r0 = threadIdx.x / CPR;   // 8 rows per pass over the threads
#pragma unroll
        for (int u = 0; u < PX; ++u) {
            const long t = min(tok0 + r0 + u * 8, (long)N - 1);
            px[u] = reinterpret_cast<const uint4*>(X + (size_t)t * d + c0)[c];
        }
#pragma unroll
        for (int u = 0; u < PW; ++u) {
            const int ge = min(eb0 + r0 + u * 8, E - 1);
            pw[u] = reinterpret_cast<const uint4*>(WgT + (size_t)ge * d + c0)[c];
        }
    };
    auto stash = [&](int eb0, int c0) {          // (rows of experts past E: zeros)
        const int cpr = min(DC, d - c0) / V;
        const int c = threadIdx.x & (CPR - 1), r0 = threadIdx.x / CPR;
        if (c < cpr) {
#pragma unroll
            for (int u = 0; u < PX; ++u) *reinterpret_cast<uint4*>(sX + (r0 + u * 8) * S + c * V) = by_value(px[u]);
#pragma unroll
            for (int u = 0; u < PW; ++u)
                *reinterpret_cast<uint4*>(sW + (r0 + u * 8) * S + c * V) = eb0 + r0 + u * 8 < E ? pw[u] : make_uint4(0, 0, 0, 0);
        }
    };

    double v[kMaxK];
    int id[kMaxK];
#pragma unroll
    for (int j = 0; j < kMaxK; ++j) { v[j] = ninf; id[j] = 0x7fffffff; }
    const T* xa = sX + (lane & 15) * S + (lane >> 4) * 8;
    const T* wb = sW + (wave * 16 + (lane & 15)) * S + (lane >> 4) * 8;

    fetch(0, 0);
    for (int blk = 0; blk < nblk; ++blk) {
        const int eb0 = blk * 64;
        const bool mine = eb0 + wave * 16 < E;       // (wave-uniform) this wavefront's 16 experts exist
        f64x4 acc[MT][CH];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int ch = 0; ch < CH; ++ch) acc[mt][ch] = f64x4{0.0, 0.0, 0.0, 0.0};
        for (int sl = 0; sl < nslab; ++sl) {
            const int c0 = sl * DC;
            __syncthreads();                         // previous slab (or the logit patch) fully consumed
            stash(eb0, c0);
            __syncthreads();
            if (sl + 1 < nslab) fetch(eb0, c0 + DC);
            else if (blk + 1 < nblk) fetch(eb0 + 64, 0);
            const int ngrp = mine ? min(DC, d - c0) / 32 : 0;
            for (int grp = 0; grp < ngrp; ++grp) {
                uint4 wt[Piece<T>::N], xt[MT][Piece<T>::N];
#pragma unroll
                for (int q = 0; q < Piece<T>::N; ++q) {
                    wt[q] = reinterpret_cast<const uint4*>(wb + grp * 32)[q];
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) xt[mt][q] = reinterpret_cast<const uint4*>(xa + mt * 16 * S + grp * 32)[q];
                }
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const double b = Piece<T>::get(wt, j);
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
                        acc[mt][j % CH] = __builtin_amdgcn_mfma_f64_16x16x4f64(Piece<T>::get(xt[mt], j), b, acc[mt][j % CH], 0, 0, 0);
                }
            }
        }
        // ---- the block's logits: through LDS, then token-per-lane into this wavefront's sorted k-list ----
        __syncthreads();                             // all waves are done with the slabs
        double* sL = reinterpret_cast<double*>(smem_raw);   // [TT tokens][64 experts]
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                double l = acc[mt][0][r];
                if constexpr (CH == 2) l += acc[mt][CH - 1][r];
                sL[(mt * 16 + 4 * r + (lane >> 4)) * 64 + wave * 16 + (lane & 15)] = l;
            }
        __syncthreads();
        for (int e = 0; e < 16; ++e) {               // lane = token (lanes past TT repeat the work of lane % TT)
            const int ge = eb0 + wave * 16 + e;
            if (ge < E) {                            // wave-uniform
                double l = sL[(lane % TT) * 64 + wave * 16 + e] + (bg ? (double)bg[ge] : 0.0);
                if (!(l == l)) l = ninf;             // NaN ranks last; indices stay in range
                if (logits_out && lane < TT && tok0 + lane < N) logits_out[(size_t)(tok0 + lane) * E + ge] = l;
                topk_insert(l, ge, v, id, k);
            }
        }
    }
    // merge the four per-wavefront lists
    __syncthreads();
    double* mV = reinterpret_cast<double*>(smem_raw);        // [wave][slot][lane]
    int* mI = reinterpret_cast<int*>(mV + 4 * kMaxK * 64);
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
        if (lane < TT && t < N) {
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

template <typename T, int MT>
static void launch_wide_mt(const moe_desc_t& D, const T* X, const T* WgT, const float* bg, int32_t* idx, float* w,
                           double* logits, hipStream_t st)
{
    constexpr int S = 512 / (int)sizeof(T) + 16 / (int)sizeof(T);
    constexpr int slab = (16 * MT + 64) * S * (int)sizeof(T), merge = 4 * kMaxK * 64 * (8 + 4);
    constexpr int smem = slab > merge ? slab : merge;      // the logit patch (16*MT x 64 doubles) is smaller than the slabs
    auto kern = gate_mfma_wide_kernel<T, MT>;
    if (!allow_dynamic_lds(kern, smem)) return;
    hipLaunchKernelGGL(kern, dim3((unsigned)((D.N + 16 * MT - 1) / (16 * MT))), dim3(256), smem, st, X, WgT, bg, D.N, D.d,
                       D.E, D.k, idx, w, logits);
}

template <typename T>
static void launch_mfma(const moe_desc_t& D, const T* X, const T* Wg, const float* bg, int32_t* idx, float* w, T* WgT,
                        double* logits, hipStream_t st)
{
    if (D.E <= 32) {
        hipLaunchKernelGGL((gate_mfma_kernel<T, 2>), dim3((unsigned)((D.N + 63) / 64)), dim3(256), 0, st, X, Wg, bg, D.N, D.d,
                           D.E, D.k, idx, w, logits);
        return;
    }
    const long n = (long)D.d * D.E;
    hipLaunchKernelGGL(gate_transpose<T>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, Wg, WgT, D.d, D.E);
    // as many tokens per workgroup as still leave two workgroups for every compute unit (one wavefront per SIMD
    // and workgroup: the second workgroup fills the matrix cores while the first stages a slab or waits)
    if (D.N >= 64 * 512) launch_wide_mt<T, 4>(D, X, WgT, bg, idx, w, logits, st);
    else if (D.N >= 32 * 512) launch_wide_mt<T, 2>(D, X, WgT, bg, idx, w, logits, st);
    else launch_wide_mt<T, 1>(D, X, WgT, bg, idx, w, logits, st);
}

// One wavefront per token sums exp(l - top) over the stored logits (lanes stride the experts, then a fixed
// butterfly) and keeps log-sum-exp for the backward pass and the load-balance monitor; with scores taken from the
// softmax over all E logits (rewrite) it also replaces the k scores.
__global__ __launch_bounds__(256) void gate_scores_all(const double* __restrict__ logits, const int32_t* __restrict__ topk_idx,
                                                       int N, int E, int k, float* __restrict__ topk_w,
                                                       double* __restrict__ lse, int rewrite)
{
    const int lane = threadIdx.x & 63;
    const long t = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= N) return;
    const double* l = logits + (size_t)t * E;
    const double top = l[topk_idx[t * k]];           // slot 0 holds the largest logit
    double s = 0.0;
    for (int e = lane; e < E; e += 64) s += exp(l[e] - top);
    for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
    if (rewrite && lane < k) topk_w[t * k + lane] = (float)(exp(l[topk_idx[t * k + lane]] - top) / s);
    if (lane == 0) lse[t] = top + log(s);
}

void launch_gate_topk(const moe_desc_t& D, const void* X, const void* Wg, const float* bg, int32_t* topk_idx,
                      float* topk_w, void* WgT, double* logits, double* lse, int32_t* gate_fail, hipStream_t st)
{
    if (D.dtype == MOE_BF16 && D.E > 16 && D.E <= 256 && !logits) {
        launch_gate_bf16(D, X, Wg, bg, topk_idx, topk_w, WgT, gate_fail, st);
        return;
    }
    if (D.dtype == MOE_BF16) {
        using T = unsigned short;
        if (D.E <= 16) launch_mfma16<T>(D, (const T*)X, (const T*)Wg, bg, topk_idx, topk_w, logits, st);
        else launch_mfma<T>(D, (const T*)X, (const T*)Wg, bg, topk_idx, topk_w, (T*)WgT, logits, st);
    } else {
        using T = float;
        if (D.E <= 16) launch_mfma16<T>(D, (const T*)X, (const T*)Wg, bg, topk_idx, topk_w, logits, st);
        else launch_mfma<T>(D, (const T*)X, (const T*)Wg, bg, topk_idx, topk_w, (T*)WgT, logits, st);
    }
    if (logits)
        hipLaunchKernelGGL(gate_scores_all, dim3((unsigned)((D.N + 3) / 4)), dim3(256), 0, st, (const double*)logits,
                           (const int32_t*)topk_idx, D.N, D.E, D.k, topk_w, lse, D.score_all);
}

}  // namespace moe
