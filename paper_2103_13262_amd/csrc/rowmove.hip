// Row-movement kernels around the expert matrix products (Section 4: "scatter" puts the
// samples of one expert into contiguous memory, "gather" puts the rows back in their original
// order; Algorithm 1: y accumulates score_i * E_i(x)), and their gradients.  All are bound by
// HBM traffic: every thread moves 16-byte pieces of a row, rows are addressed through pos/perm.
#include "common.h"

namespace moe {

// 16 bytes of a row as floats: 8 bf16 or 4 fp32 elements.
template <typename T> struct Vec;
template <> struct Vec<unsigned short> {
    static constexpr int N = 8;
    static __device__ __forceinline__ void load(const void* base, size_t chunk, float* f)
    {
        const uint4 v = ((const uint4*)base)[chunk];
        const unsigned w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = __uint_as_float(w[i] << 16);
            f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
    static __device__ __forceinline__ void store(void* base, size_t chunk, const float* f)
    {
        unsigned w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) w[i] = pack_bf16x2(f[2 * i], f[2 * i + 1]);
        ((uint4*)base)[chunk] = make_uint4(w[0], w[1], w[2], w[3]);
    }
};
template <> struct Vec<float> {
    static constexpr int N = 4;
    static __device__ __forceinline__ void load(const void* base, size_t chunk, float* f)
    {
        const float4 v = ((const float4*)base)[chunk];
        f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
    }
    static __device__ __forceinline__ void store(void* base, size_t chunk, const float* f)
    {
        ((float4*)base)[chunk] = make_float4(f[0], f[1], f[2], f[3]);
    }
};

// ---- scatter: Xs[r,:] = X[perm[r] / k, :] ------------------------------------------------------
__global__ __launch_bounds__(256) void scatter_rows(const uint4* __restrict__ X, const int32_t* __restrict__ perm,
                                                    uint4* __restrict__ Xs, long M, int k, int cpr)
{
    const long total = M * cpr;
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long)gridDim.x * 256) {
        const long r = i / cpr;
        const int c = (int)(i - r * cpr);
        const long t = perm[r] / k;
        Xs[i] = X[t * cpr + c];
    }
}

// ---- combine: Y[t,:] = sum_j w[t,j] * Ys[pos[t*k+j], :]  (slots in ascending j, fp32) ---------
template <typename T>
__global__ __launch_bounds__(256) void combine_rows(const void* __restrict__ Ys, const float* __restrict__ topk_w,
                                                    const int32_t* __restrict__ pos, void* __restrict__ Y, long N,
                                                    int k, int cpr)
{
    constexpr int V = Vec<T>::N;
    const long total = N * cpr;
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long)gridDim.x * 256) {
        const long t = i / cpr;
        const int c = (int)(i - t * cpr);
        float acc[V];
#pragma unroll
        for (int u = 0; u < V; ++u) acc[u] = 0.f;
        for (int j = 0; j < k; ++j) {
            const long a = t * k + j;
            const float w = topk_w[a];
            float v[V];
            Vec<T>::load(Ys, (size_t)pos[a] * cpr + c, v);
#pragma unroll
            for (int u = 0; u < V; ++u) acc[u] = fmaf(w, v[u], acc[u]);
        }
        Vec<T>::store(Y, (size_t)i, acc);
    }
}

// ---- combine backward: one wavefront per token -------------------------------------------------
//   dYs[pos[a],:] = w[a] * dY[t,:];  dw[a] = <dY[t,:], Ys[pos[a],:]>;  dl_j = w_j (dw_j - sum_i w_i dw_i)
//   (Ys == NULL: the expert outputs were not kept - top-1 with the score fixed at 1, where dl is exactly zero)
//   Rides along (X != NULL): Xs[pos[a],:] = X[t,:], the scatter that the weight gradients of the first layer and of
//   the gate read; the token's row is in hand anyway, and the backward pass saves a launch.
template <typename T>
__global__ __launch_bounds__(256) void dcombine_rows(const void* __restrict__ dY, const void* __restrict__ Ys,
                                                     const float* __restrict__ topk_w,
                                                     const int32_t* __restrict__ pos, void* __restrict__ dYs,
                                                     float* __restrict__ dl, long N, int k, int cpr,
                                                     float* __restrict__ S_out,   // S_out: sum_i w_i dw_i per token, or NULL
                                                     const uint4* __restrict__ X, uint4* __restrict__ Xs)
{
    constexpr int V = Vec<T>::N;
    const int lane = threadIdx.x & 63;
    const long t = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= N) return;
    float w[kMaxK], dw[kMaxK];
    size_t r[kMaxK];
#pragma unroll
    for (int j = 0; j < kMaxK; ++j) {
        dw[j] = 0.f;
        if (j < k) { r[j] = (size_t)pos[t * k + j]; w[j] = topk_w[t * k + j]; }
    }
    for (int c = lane; c < cpr; c += 64) {
        float g[V];
        Vec<T>::load(dY, (size_t)t * cpr + c, g);
        uint4 x = make_uint4(0, 0, 0, 0);
        if (X) x = X[(size_t)t * cpr + c];
#pragma unroll
        for (int j = 0; j < kMaxK; ++j) {
            if (j >= k) break;
            float y[V], o[V];
            if (Ys) Vec<T>::load(Ys, r[j] * cpr + c, y);
            else {
#pragma unroll
                for (int u = 0; u < V; ++u) y[u] = 0.f;
            }
#pragma unroll
            for (int u = 0; u < V; ++u) {
                o[u] = w[j] * g[u];
                dw[j] = fmaf(g[u], y[u], dw[j]);
            }
            Vec<T>::store(dYs, r[j] * cpr + c, o);
            if (X) Xs[r[j] * cpr + c] = x;
        }
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < kMaxK; ++j) {
        if (j >= k) break;
        float part = dw[j];
        for (int off = 32; off > 0; off >>= 1) part += __shfl_xor(part, off, 64);
        dw[j] = part;
        s = fmaf(w[j], part, s);
    }
    if (lane == 0) {
#pragma unroll
        for (int j = 0; j < kMaxK; ++j)
            if (j < k) dl[t * k + j] = w[j] * (dw[j] - s);
        if (S_out) S_out[t] = s;
    }
}

// ---- dX[t,:] = sum_j dXs[pos[a],:] + sum_j dl[a] * Wg[:, idx[a]] ------------------------------
template <typename T>
__device__ __forceinline__ void gate_bwd_dx_body(long block, long blocks, const void* __restrict__ dXs, const void* __restrict__ WgT,
                                                 const float* __restrict__ dl, const int32_t* __restrict__ topk_idx,
                                                 const int32_t* __restrict__ pos, void* __restrict__ dX, long N, int k,
                                                 int cpr, const float* __restrict__ dxd)   // dxd: [N][d] float to add, or NULL
{
    constexpr int V = Vec<T>::N;
    const long total = N * cpr;
    for (long i = block * 256 + threadIdx.x; i < total; i += blocks * 256) {
        const long t = i / cpr;
        const int c = (int)(i - t * cpr);
        float acc[V];
#pragma unroll
        for (int u = 0; u < V; ++u) acc[u] = 0.f;
        for (int j = 0; j < k; ++j) {
            float v[V];
            Vec<T>::load(dXs, (size_t)pos[t * k + j] * cpr + c, v);
#pragma unroll
            for (int u = 0; u < V; ++u) acc[u] += v[u];
        }
        for (int j = 0; j < k; ++j) {
            const long a = t * k + j;
            const float g = dl[a];
            float wv[V];
            Vec<T>::load(WgT, (size_t)topk_idx[a] * cpr + c, wv);
#pragma unroll
            for (int u = 0; u < V; ++u) acc[u] = fmaf(g, wv[u], acc[u]);
        }
        if (dxd) {
#pragma unroll
            for (int u = 0; u < V; ++u) acc[u] += dxd[(size_t)i * V + u];
        }
        Vec<T>::store(dX, (size_t)i, acc);
    }
}

// ---- dWg[:,e] = sum over rows r of segment e of dl[perm[r]] * Xs[r,:]  (fixed order) ----------
// Every expert's segment is cut into pieces of 64 rows (the 64-row tile table of the plan step), so the
// work per workgroup is the same however skewed the load is.  grid (max pieces, ceil(cpr/64)); each thread
// owns one 16-byte column piece and walks the rows of its piece; a second kernel adds an expert's pieces
// in ascending order.
template <typename T>
__global__ __launch_bounds__(512) void dwg_partial(const void* __restrict__ Xs, const float* __restrict__ dl,
                                                   const int32_t* __restrict__ perm, const int32_t* __restrict__ counts,
                                                   const int32_t* __restrict__ offsets, const int32_t* __restrict__ P64,
                                                   float* __restrict__ part, float* __restrict__ bpart, int E, int d,
                                                   int cpr, const T* __restrict__ Wg, T* __restrict__ WgT)
{
    // Rides along (WgT != nullptr): WgT[e][i] = Wg[i][e], which lets the kernel that follows the reduction read a
    // gate column as contiguous 16-byte pieces; spread over all workgroups of the launch.
    if (WgT) {
        const long nel = (long)d * E, nthr = (long)gridDim.x * gridDim.y * 512;
        for (long i = ((long)blockIdx.y * gridDim.x + blockIdx.x) * 512 + threadIdx.x; i < nel; i += nthr) {
            const int ee = (int)(i / d), row = (int)(i - (long)ee * d);
            WgT[i] = Wg[(size_t)row * E + ee];
        }
    }
    // 64 column threads x 8 row groups: group q walks rows 8q .. 8q+7 of the piece (all eight loads in flight); the
    // groups' sums are added in the order (((0 + 1) + 2) + ...) + 7, so the result does not depend on timing.
    constexpr int V = Vec<T>::N;
    __shared__ float s_g[64];
    __shared__ float s_acc[7][64][V];
    const int piece = blockIdx.x;
    if (piece >= P64[E]) return;          // uniform over the workgroup
    int lo = 0, hi = E;                   // largest e with P64[e] <= piece
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (P64[mid] <= piece) lo = mid; else hi = mid;
    }
    const int e = lo;
    const int r0 = offsets[e] + (piece - P64[e]) * 64;
    const int r1 = min(r0 + 64, offsets[e] + counts[e]);
    // (dl == nullptr: plain column sums of the segment, every row with weight 1: the expert-bias gradients)
    if (threadIdx.x < 64) s_g[threadIdx.x] = r0 + (int)threadIdx.x < r1 ? (dl ? dl[perm[r0 + threadIdx.x]] : 1.f) : 0.f;
    __syncthreads();
    const int ct = threadIdx.x & 63, q = threadIdx.x >> 6;
    const int c = blockIdx.y * 64 + ct;
    const bool active = c < cpr;
    float acc[V];
#pragma unroll
    for (int u = 0; u < V; ++u) acc[u] = 0.f;
    if (active) {
        float v[8][V];
#pragma unroll
        for (int i = 0; i < 8; ++i) {         // rows past the end of the piece contribute g = 0; their loads are skipped
            const int r = r0 + q * 8 + i;
#pragma unroll
            for (int u = 0; u < V; ++u) v[i][u] = 0.f;
            if (r < r1) Vec<T>::load(Xs, (size_t)r * cpr + c, v[i]);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float g = s_g[q * 8 + i];
#pragma unroll
            for (int u = 0; u < V; ++u) acc[u] = fmaf(g, v[i][u], acc[u]);
        }
    }
    if (q > 0) {
#pragma unroll
        for (int u = 0; u < V; ++u) s_acc[q - 1][ct][u] = acc[u];
    }
    __syncthreads();
    if (q == 0 && active) {
#pragma unroll
        for (int g = 0; g < 7; ++g)
#pragma unroll
            for (int u = 0; u < V; ++u) acc[u] += s_acc[g][ct][u];
        float* dst = part + (size_t)piece * d + (size_t)c * V;
#pragma unroll
        for (int u = 0; u < V; ++u) dst[u] = acc[u];
        if (c == 0 && bpart) {
            float sdl = 0.f;
            for (int i = 0; i < 64; ++i) sdl += s_g[i];
            bpart[piece] = sdl;
        }
    }
}

// grid (ceil(d / 256), E): a thread owns one row of one expert's column, so that the threads of a wavefront read
// consecutive floats of every piece; the pieces are added in ascending order (loads four at a time, sums in order).
template <typename G>
__device__ __forceinline__ void dwg_final_body(int bx, int e, const float* __restrict__ part, const float* __restrict__ bpart,
                                               const int32_t* __restrict__ P64, G* __restrict__ dWg,
                                               float* __restrict__ dbg, int d, int E, int accumulate,
                                               const float* __restrict__ dense_part,     // [nch][E][d] to add, or NULL
                                               const float* __restrict__ dense_bpart, int nch)
{
    const int row = bx * 256 + threadIdx.x;
    const int q1 = P64[e + 1];
    if (row < d) {
        float s = 0.f;
        int q = P64[e];
        for (; q + 4 <= q1; q += 4) {
            const float a0 = part[(size_t)q * d + row], a1 = part[(size_t)(q + 1) * d + row];
            const float a2 = part[(size_t)(q + 2) * d + row], a3 = part[(size_t)(q + 3) * d + row];
            s = (((s + a0) + a1) + a2) + a3;
        }
        for (; q < q1; ++q) s += part[(size_t)q * d + row];
        if (dense_part)
            for (int c = 0; c < nch; ++c) s += dense_part[((size_t)c * E + e) * d + row];
        const size_t i = (size_t)row * E + e;
        if constexpr (sizeof(G) == 2) {
            if (accumulate) s += bf16_to_f32(dWg[i]);
            dWg[i] = f32_to_bf16(s);
        } else {
            if (accumulate) s += dWg[i];
            dWg[i] = s;
        }
    }
    if (dbg && row == 0) {
        float s = 0.f;
        for (int q = P64[e]; q < q1; ++q) s += bpart[q];
        if (dense_bpart)
            for (int c = 0; c < nch; ++c) s += dense_bpart[(size_t)c * E + e];
        if (accumulate) s += dbg[e];
        dbg[e] = s;
    }
}

// The two kernels that follow the partial sums of the gate-matrix gradient, in one launch: the first fgx * E
// workgroups add every expert's pieces (dWg, dbg), the others write dX.  Neither reads what the other writes.
template <typename T, typename G>
__global__ __launch_bounds__(256) void gate_bwd_tail(int fgx, const float* __restrict__ part, const float* __restrict__ bpart,
                                                     const int32_t* __restrict__ P64, G* __restrict__ dWg, float* __restrict__ dbg,
                                                     int d, int E, int accumulate, const float* __restrict__ dense_part,
                                                     const float* __restrict__ dense_bpart, int nch,
                                                     const void* __restrict__ dXs, const void* __restrict__ WgT,
                                                     const float* __restrict__ dl, const int32_t* __restrict__ topk_idx,
                                                     const int32_t* __restrict__ pos, void* __restrict__ dX, long N, int k, int cpr,
                                                     const float* __restrict__ dxd)
{
    const int nfinal = fgx * E;
    if ((int)blockIdx.x < nfinal)
        dwg_final_body<G>((int)blockIdx.x % fgx, (int)blockIdx.x / fgx, part, bpart, P64, dWg, dbg, d, E, accumulate, dense_part,
                          dense_bpart, nch);
    else
        gate_bwd_dx_body<T>((long)blockIdx.x - nfinal, (long)gridDim.x - nfinal, dXs, WgT, dl, topk_idx, pos, dX, N, k, cpr, dxd);
}

// out[e][c] = sum of the pieces of expert e, in ascending order (the column sums of its segment).
__global__ __launch_bounds__(256) void segsum_final(const float* __restrict__ part, const int32_t* __restrict__ P64,
                                                    float* __restrict__ out, int width, int accumulate)
{
    const int c = blockIdx.x * 256 + threadIdx.x, e = blockIdx.y;
    if (c >= width) return;
    float s = 0.f;
    for (int q = P64[e]; q < P64[e + 1]; ++q) s += part[(size_t)q * width + c];
    const size_t o = (size_t)e * width + c;
    out[o] = accumulate ? out[o] + s : s;
}

// ---- launchers -----------------------------------------------------------------------------------
static unsigned grid_for(long items)
{
    long g = (items + 255) / 256;
    if (g < 1) g = 1;
    if (g > 256 * 32) g = 256 * 32;
    return (unsigned)g;
}

void launch_scatter(const moe_desc_t& D, const void* X, const int32_t* perm, void* Xs, hipStream_t st)
{
    const long M = (long)D.N * D.k;
    const int cpr = (int)((size_t)D.d * dtype_size(D.dtype) / 16);
    hipLaunchKernelGGL(scatter_rows, dim3(grid_for(M * cpr)), dim3(256), 0, st, (const uint4*)X, perm, (uint4*)Xs, M,
                       D.k, cpr);
}

void launch_combine(const moe_desc_t& D, const void* Ys, const float* topk_w, const int32_t* pos, void* Y,
                    hipStream_t st)
{
    const int cpr = (int)((size_t)D.d * dtype_size(D.dtype) / 16);
    const unsigned g = grid_for((long)D.N * cpr);
    if (D.dtype == MOE_BF16)
        hipLaunchKernelGGL(combine_rows<unsigned short>, dim3(g), dim3(256), 0, st, Ys, topk_w, pos, Y, (long)D.N, D.k, cpr);
    else
        hipLaunchKernelGGL(combine_rows<float>, dim3(g), dim3(256), 0, st, Ys, topk_w, pos, Y, (long)D.N, D.k, cpr);
}

void launch_dcombine(const moe_desc_t& D, const void* dY, const void* Ys, const float* topk_w,
                     const int32_t* pos, void* dYs, float* dl, float* S_out, const void* X, void* Xs, hipStream_t st)
{
    const int cpr = (int)((size_t)D.d * dtype_size(D.dtype) / 16);
    const unsigned g = (unsigned)((D.N + 3) / 4);
    if (D.dtype == MOE_BF16)
        hipLaunchKernelGGL(dcombine_rows<unsigned short>, dim3(g), dim3(256), 0, st, dY, Ys, topk_w, pos, dYs, dl,
                           (long)D.N, D.k, cpr, S_out, (const uint4*)X, (uint4*)Xs);
    else
        hipLaunchKernelGGL(dcombine_rows<float>, dim3(g), dim3(256), 0, st, dY, Ys, topk_w, pos, dYs, dl, (long)D.N,
                           D.k, cpr, S_out, (const uint4*)X, (uint4*)Xs);
}

void launch_gate_bwd(const moe_desc_t& D, const WsLayout& L, const void* Xs, const void* dXs, const void* Wg,
                     const float* dl, const int32_t* topk_idx, const int32_t* pos, const int32_t* perm,
                     const int32_t* counts, const int32_t* offsets, void* dX, void* dWg, float* dbg, char* ws,
                     const void* X_dense, hipStream_t st)
{
    // X_dense != NULL (scores over all experts): the experts that were not selected receive gradient too; their
    // dense terms are computed first and added inside the kernels below that round dWg, dbg and dX.
    const float *dpart = nullptr, *dbpart = nullptr, *dxd = nullptr;
    if (X_dense) {
        launch_gate_dense(D, L, X_dense, Wg, topk_idx, ws, st);
        dpart = (const float*)(ws + L.dense_part);
        dbpart = (const float*)(ws + L.dense_bpart);
        if (D.N > 0) dxd = (const float*)(ws + L.dx_dense);
    }
    const int nch = D.N > 0 ? L.dense_chunks : 0;
    const int cpr = (int)((size_t)D.d * dtype_size(D.dtype) / 16);
    float* part = (float*)(ws + L.dwg_part);
    float* bpart = (float*)(ws + L.dbg_part);
    const int32_t* P64 = (const int32_t*)(ws + L.tileP) + tile_height_index(64) * (D.E + 1);
    const dim3 pg((unsigned)L.dwg_pieces, (cpr + 63) / 64);
    const unsigned xg = grid_for((long)D.N * cpr);
    void* WgT = ws + L.WgT;
    const int fgx = (D.d + 255) / 256;
    const dim3 tg((unsigned)(fgx * D.E) + xg);
    if (D.dtype == MOE_BF16) {
        using T = unsigned short;
        hipLaunchKernelGGL(dwg_partial<T>, pg, dim3(512), 0, st, Xs, dl, perm, counts, offsets, P64, part, bpart, D.E, D.d, cpr,
                           (const T*)Wg, (T*)WgT);
        if (D.grad_dtype == MOE_BF16)
            hipLaunchKernelGGL((gate_bwd_tail<T, unsigned short>), tg, dim3(256), 0, st, fgx, (const float*)part, (const float*)bpart, P64,
                               (unsigned short*)dWg, dbg, D.d, D.E, D.accumulate, dpart, dbpart, nch, dXs, (const void*)WgT, dl,
                               topk_idx, pos, dX, (long)D.N, D.k, cpr, dxd);
        else
            hipLaunchKernelGGL((gate_bwd_tail<T, float>), tg, dim3(256), 0, st, fgx, (const float*)part, (const float*)bpart, P64,
                               (float*)dWg, dbg, D.d, D.E, D.accumulate, dpart, dbpart, nch, dXs, (const void*)WgT, dl, topk_idx,
                               pos, dX, (long)D.N, D.k, cpr, dxd);
    } else {
        using T = float;
        hipLaunchKernelGGL(dwg_partial<T>, pg, dim3(512), 0, st, Xs, dl, perm, counts, offsets, P64, part, bpart, D.E, D.d, cpr,
                           (const T*)Wg, (T*)WgT);
        hipLaunchKernelGGL((gate_bwd_tail<T, float>), tg, dim3(256), 0, st, fgx, (const float*)part, (const float*)bpart, P64,
                           (float*)dWg, dbg, D.d, D.E, D.accumulate, dpart, dbpart, nch, dXs, (const void*)WgT, dl, topk_idx, pos,
                           dX, (long)D.N, D.k, cpr, dxd);
    }
}

// out[E][width] (float) = column sums of src[M][width] over every expert's segment (fixed order).
void launch_segment_sums(const moe_desc_t& D, const WsLayout& L, const void* src, int width, const int32_t* counts,
                         const int32_t* offsets, float* out, char* ws, hipStream_t st)
{
    const int cpr = (int)((size_t)width * dtype_size(D.dtype) / 16);
    float* part = (float*)(ws + L.bias_part);
    const int32_t* P64 = (const int32_t*)(ws + L.tileP) + tile_height_index(64) * (D.E + 1);
    const dim3 pg((unsigned)L.dwg_pieces, (cpr + 63) / 64);
    if (D.dtype == MOE_BF16)
        hipLaunchKernelGGL(dwg_partial<unsigned short>, pg, dim3(512), 0, st, src, (const float*)nullptr,
                           (const int32_t*)nullptr, counts, offsets, P64, part, (float*)nullptr, D.E, width, cpr,
                           (const unsigned short*)nullptr, (unsigned short*)nullptr);
    else
        hipLaunchKernelGGL(dwg_partial<float>, pg, dim3(512), 0, st, src, (const float*)nullptr, (const int32_t*)nullptr,
                           counts, offsets, P64, part, (float*)nullptr, D.E, width, cpr, (const float*)nullptr, (float*)nullptr);
    hipLaunchKernelGGL(segsum_final, dim3((unsigned)((width + 255) / 256), (unsigned)D.E), dim3(256), 0, st,
                       (const float*)part, P64, out, width, D.accumulate);
}

}  // namespace moe
