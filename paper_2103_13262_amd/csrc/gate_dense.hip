// Gate gradient of the experts that were NOT selected, for scores taken from the softmax over all experts
// (desc.score_all; Algorithm 1 with a softmax gate, Section 2.1: the gate is trained through the score).
// With p = softmax(l) and S = sum_j w_j dL/dw_j over a token's slots, an expert b outside the selection has
// dL/dl_b = -p_b S.  These terms are dense in (token, expert), so they are handled as two small dense products
// beside the sparse kernels of the selected experts:
//   R[t][e]      = -exp(l[t][e] - lse[t]) S[t], 0 at the selected experts                     (gate_dense_r)
//   dWg[:, e]   += sum_t X[t][:] R[t][e],  dbg[e] += sum_t R[t][e]   by chunks of 512 tokens   (dense_dwg_partial)
//   dX[t][:]    += sum_e R[t][e] Wg[:, e]                                                      (dense_dx)
// Both are fp32 FMA kernels on 64 x 64 tiles staged in LDS, summed in a fixed order; their results are added inside
// the kernels that round dWg and dX, so each output is rounded once.
#include "common.h"

namespace moe {

namespace {
template <typename T> __device__ __forceinline__ float to_f32(T v);
template <> __device__ __forceinline__ float to_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f32<unsigned short>(unsigned short v) { return bf16_to_f32(v); }

constexpr int kTile = 64, kPitch = kTile + 4;
}  // namespace

__global__ __launch_bounds__(256) void gate_dense_r(const double* __restrict__ logits, const double* __restrict__ lse,
                                                    const float* __restrict__ S, const int32_t* __restrict__ topk_idx,
                                                    long N, int E, int k, float* __restrict__ R)
{
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i >= N * E) return;
    const long t = i / E;
    const int e = (int)(i - t * E);
    bool sel = false;
    for (int j = 0; j < k; ++j) sel |= topk_idx[t * k + j] == e;
    R[i] = sel ? 0.f : (float)(-exp(logits[i] - lse[t]) * (double)S[t]);
}

// grid (chunks of 512 tokens, d / 64, ceil(E / 64)); part[c][e][i], bpart[c][e]
template <typename T>
__global__ __launch_bounds__(256) void dense_dwg_partial(const T* __restrict__ X, const float* __restrict__ R, long N, int d,
                                                         int E, float* __restrict__ part, float* __restrict__ bpart)
{
    __shared__ float sX[kTile][kPitch];   // [token][feature]
    __shared__ float sR[kTile][kPitch];   // [token][expert]
    const int c = blockIdx.x, i0 = blockIdx.y * kTile, e0 = blockIdx.z * kTile;
    const int ti = threadIdx.x >> 4, te = threadIdx.x & 15;
    float acc[4][4] = {}, bsum[4] = {0.f, 0.f, 0.f, 0.f};
    for (int sub = 0; sub < 8; ++sub) {
        const long t0 = (long)c * 512 + sub * kTile;
        if (t0 >= N) break;                       // uniform
        __syncthreads();
        for (int q = threadIdx.x; q < kTile * kTile; q += 256) {
            const int tt = q >> 6, x = q & 63;
            const long t = t0 + tt;
            sX[tt][x] = (t < N && i0 + x < d) ? to_f32<T>(X[(size_t)t * d + i0 + x]) : 0.f;
            sR[tt][x] = (t < N && e0 + x < E) ? R[(size_t)t * E + e0 + x] : 0.f;
        }
        __syncthreads();
#pragma unroll 8
        for (int tt = 0; tt < kTile; ++tt) {
            const float4 xv = *reinterpret_cast<const float4*>(&sX[tt][ti * 4]);
            const float4 rv = *reinterpret_cast<const float4*>(&sR[tt][te * 4]);
            const float x[4] = {xv.x, xv.y, xv.z, xv.w}, r[4] = {rv.x, rv.y, rv.z, rv.w};
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = 0; b < 4; ++b) acc[a][b] = fmaf(x[a], r[b], acc[a][b]);
#pragma unroll
            for (int b = 0; b < 4; ++b) bsum[b] += r[b];
        }
    }
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        const int e = e0 + te * 4 + b;
        if (e >= E) continue;
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            const int i = i0 + ti * 4 + a;
            if (i < d) part[((size_t)c * E + e) * d + i] = acc[a][b];
        }
        if (blockIdx.y == 0 && ti == 0) bpart[(size_t)c * E + e] = bsum[b];
    }
}

// grid (ceil(N / 64), d / 64); dxd[t][i] = sum_e R[t][e] Wg[i][e]
template <typename T>
__global__ __launch_bounds__(256) void dense_dx(const float* __restrict__ R, const T* __restrict__ Wg, long N, int d, int E,
                                                float* __restrict__ dxd)
{
    __shared__ float sRt[kTile][kPitch];  // [expert][token]
    __shared__ float sW[kTile][kPitch];   // [expert][feature]
    const long t0 = (long)blockIdx.x * kTile;
    const int i0 = blockIdx.y * kTile;
    const int ti = threadIdx.x >> 4, tf = threadIdx.x & 15;
    float acc[4][4] = {};
    for (int e0 = 0; e0 < E; e0 += kTile) {
        __syncthreads();
        for (int q = threadIdx.x; q < kTile * kTile; q += 256) {
            const int a = q >> 6, ee = q & 63;          // ee runs fastest: both sources are contiguous in e
            sRt[ee][a] = (t0 + a < N && e0 + ee < E) ? R[(size_t)(t0 + a) * E + e0 + ee] : 0.f;
            sW[ee][a] = (i0 + a < d && e0 + ee < E) ? to_f32<T>(Wg[(size_t)(i0 + a) * E + e0 + ee]) : 0.f;
        }
        __syncthreads();
#pragma unroll 8
        for (int ee = 0; ee < kTile; ++ee) {
            const float4 rv = *reinterpret_cast<const float4*>(&sRt[ee][ti * 4]);
            const float4 wv = *reinterpret_cast<const float4*>(&sW[ee][tf * 4]);
            const float r[4] = {rv.x, rv.y, rv.z, rv.w}, w[4] = {wv.x, wv.y, wv.z, wv.w};
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = 0; b < 4; ++b) acc[a][b] = fmaf(r[a], w[b], acc[a][b]);
        }
    }
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        const long t = t0 + ti * 4 + a;
        if (t >= N) continue;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int i = i0 + tf * 4 + b;
            if (i < d) dxd[(size_t)t * d + i] = acc[a][b];
        }
    }
}

// ---- load-balance monitor: share of the assignments and mean gate probability of every expert ----------------
// grid (chunks of 512 tokens, ceil(E / 256)): psum[c][e] = sum over the chunk's tokens, in ascending order, of
// exp(l[t][e] - lse[t]).
__global__ __launch_bounds__(256) void balance_partial(const double* __restrict__ logits, const double* __restrict__ lse,
                                                       long N, int E, double* __restrict__ psum)
{
    const int c = blockIdx.x, e = blockIdx.y * 256 + threadIdx.x;
    if (e >= E) return;
    const long t1 = min((long)(c + 1) * 512, N);
    double s = 0.0;
    for (long t = (long)c * 512; t < t1; ++t) s += exp(logits[(size_t)t * E + e] - lse[t]);
    psum[(size_t)c * E + e] = s;
}

// one workgroup: the chunks in ascending order per expert, then the scalar over the experts in ascending order
__global__ __launch_bounds__(1024) void balance_final(const double* __restrict__ psum, const int32_t* __restrict__ counts,
                                                      long N, int E, int k, int nch, float* __restrict__ fraction,
                                                      float* __restrict__ mean_prob, float* __restrict__ loss)
{
    __shared__ double s_term[kMaxE];
    const int e = threadIdx.x;
    if (e < E) {
        double p = 0.0;
        for (int c = 0; c < nch; ++c) p += psum[(size_t)c * E + e];
        p = N > 0 ? p / (double)N : 0.0;
        const double f = N > 0 ? (double)counts[e] / ((double)N * k) : 0.0;
        if (fraction) fraction[e] = (float)f;
        if (mean_prob) mean_prob[e] = (float)p;
        s_term[e] = f * p;
    }
    __syncthreads();
    if (threadIdx.x == 0 && loss) {
        double s = 0.0;
        for (int i = 0; i < E; ++i) s += s_term[i];
        *loss = (float)(s * E);
    }
}

void launch_balance_stats(const moe_desc_t& D, const WsLayout& L, const int32_t* counts, float* fraction, float* mean_prob,
                          float* loss, char* ws, hipStream_t st)
{
    double* psum = (double*)(ws + L.prob_part);
    const int nch = D.N > 0 ? L.dense_chunks : 0;
    if (nch > 0)
        hipLaunchKernelGGL(balance_partial, dim3((unsigned)nch, (unsigned)((D.E + 255) / 256)), dim3(256), 0, st,
                           (const double*)(ws + L.logits), (const double*)(ws + L.lse), (long)D.N, D.E, psum);
    hipLaunchKernelGGL(balance_final, dim3(1), dim3(1024), 0, st, (const double*)psum, counts, (long)D.N, D.E, D.k, nch,
                       fraction, mean_prob, loss);
}

void launch_gate_dense(const moe_desc_t& D, const WsLayout& L, const void* X, const void* Wg, const int32_t* topk_idx,
                       char* ws, hipStream_t st)
{
    const double* logits = (const double*)(ws + L.logits);
    const double* lse = (const double*)(ws + L.lse);
    const float* S = (const float*)(ws + L.gate_S);
    float* R = (float*)(ws + L.gate_R);
    float* dxd = (float*)(ws + L.dx_dense);
    float* part = (float*)(ws + L.dense_part);
    float* bpart = (float*)(ws + L.dense_bpart);
    const long N = D.N;
    if (N == 0) return;
    hipLaunchKernelGGL(gate_dense_r, dim3((unsigned)((N * D.E + 255) / 256)), dim3(256), 0, st, logits, lse, S, topk_idx, N,
                       D.E, D.k, R);
    const dim3 g1((unsigned)L.dense_chunks, (unsigned)((D.d + kTile - 1) / kTile), (unsigned)((D.E + kTile - 1) / kTile));
    const dim3 g2((unsigned)((N + kTile - 1) / kTile), (unsigned)((D.d + kTile - 1) / kTile));
    if (D.dtype == MOE_BF16) {
        using T = unsigned short;
        hipLaunchKernelGGL(dense_dwg_partial<T>, g1, dim3(256), 0, st, (const T*)X, (const float*)R, N, D.d, D.E, part, bpart);
        hipLaunchKernelGGL(dense_dx<T>, g2, dim3(256), 0, st, (const float*)R, (const T*)Wg, N, D.d, D.E, dxd);
    } else {
        using T = float;
        hipLaunchKernelGGL(dense_dwg_partial<T>, g1, dim3(256), 0, st, (const T*)X, (const float*)R, N, D.d, D.E, part, bpart);
        hipLaunchKernelGGL(dense_dx<T>, g2, dim3(256), 0, st, (const float*)R, (const T*)Wg, N, D.d, D.E, dxd);
    }
}

}  // namespace moe
