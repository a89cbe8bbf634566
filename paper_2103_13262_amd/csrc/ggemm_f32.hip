// Grouped matrix products in fp32 (used when desc.dtype is fp32): the experts' fully-connected
// layers applied to their contiguous batches (Section 3.1, the dedicated linear module; Section 4)
// and the matching gradients.  Plain LDS-tiled FMA kernel: 64x64 output tile, 16-deep steps,
// 256 threads with a 4x4 micro-tile each.  One launch covers all experts; the tile -> expert map
// comes from the prefix table written by the plan step.
#include "common.h"

namespace moe {

namespace {
constexpr int TM = 64, TN = 64, TK = 16;

struct TileF32 {
    const float* A; long sam, sak;   // A'(m,kk) = A[m*sam + kk*sak]
    const float* B; long sbk, sbn;   // B'(kk,n) = B[kk*sbk + n*sbn]
    float* C; float* C2; const float* Z; const float* bias; long ldc;   // bias: the expert's row at the tile's first column, or NULL
    int Mt, Nt, Kt;                  // valid extents of this tile / reduction length
    const int32_t* gather; int div;  // rows kinds: row m of A' is A[gather[row0 + m] / div] (A then points at the base), or NULL
    const int32_t* scatter;          // kRowsNN: row m of the tile is written to row scatter[row0 + m] of C (C then points at column n0 of the base), or NULL
    long row0;
};

__global__ __launch_bounds__(256) void ggemm_f32_kernel(GemmArgs g, int ntn)
{
    __shared__ float As[TK][TM + 4];
    __shared__ float Bs[TK][TN + 4];
    TileF32 t{};
    const float* A = (const float*)g.A;
    const float* B = (const float*)g.B;
    if (g.kind == kColsT) {
        const int e = blockIdx.z;
        const int m0 = blockIdx.y * TM, n0 = blockIdx.x * TN;
        const long off = g.offsets[e];
        t.A = A + off * g.K + m0;      t.sam = 1;      t.sak = g.K;
        t.B = B + off * g.Nout + n0;   t.sbk = g.Nout; t.sbn = 1;
        t.C = (float*)g.C + ((size_t)e * g.K + m0) * g.Nout + n0;
        t.C2 = nullptr; t.Z = nullptr; t.bias = nullptr; t.ldc = g.Nout;
        t.Mt = min(TM, g.K - m0); t.Nt = min(TN, g.Nout - n0); t.Kt = g.counts[e];
    } else {
        const int32_t* P = g.tileP + tile_height_index(TM) * (g.E + 1);
        const int tile = blockIdx.x / ntn, nt = blockIdx.x % ntn;
        if (tile >= P[g.E]) return;
        int lo = 0, hi = g.E;            // largest e with P[e] <= tile
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (P[mid] <= tile) lo = mid; else hi = mid;
        }
        const int e = lo;
        const int mt = tile - P[e];
        const long r0 = (long)g.offsets[e] + (long)mt * TM;
        const int n0 = nt * TN;
        t.A = g.a_gather ? A : A + r0 * g.K; t.sam = g.K; t.sak = 1;
        t.gather = g.a_gather; t.div = g.a_gather_div; t.row0 = r0;
        t.scatter = g.kind == kRowsNN ? g.c_scatter : nullptr;
        const float* Be = B + (size_t)e * g.K * g.Nout;
        if (g.kind == kRowsNN || g.kind == kRowsNN_GeLU) { t.B = Be + n0; t.sbk = g.Nout; t.sbn = 1; }
        else { t.B = Be + (size_t)n0 * g.K; t.sbk = 1; t.sbn = g.K; }
        t.C = (float*)g.C + (t.scatter ? 0 : r0 * g.Nout) + n0;
        t.C2 = g.C2 ? (float*)g.C2 + r0 * g.Nout + n0 : nullptr;
        t.Z = g.Zin ? (const float*)g.Zin + r0 * g.Nout + n0 : nullptr;
        t.bias = g.bias && (g.kind == kRowsNN || g.kind == kRowsNN_GeLU) ? (const float*)g.bias + (size_t)e * g.Nout + n0 : nullptr;
        t.ldc = g.Nout;
        t.Mt = min(TM, g.counts[e] - mt * TM); t.Nt = min(TN, g.Nout - n0); t.Kt = g.K;
    }

    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < t.Kt; k0 += TK) {
        for (int q = threadIdx.x; q < TK * TM; q += 256) {
            const int kk = q / TM, m = q % TM;   // m fastest: for sam==1 (transposed A) reads coalesce
            const int kk2 = q % TK, m2 = q / TK; // kk fastest: for sak==1 reads coalesce
            const int K_ = t.sak == 1 ? kk2 : kk, M_ = t.sak == 1 ? m2 : m;
            float v = 0.f;
            if (M_ < t.Mt && k0 + K_ < t.Kt) {
                const long arow = t.gather ? (long)(t.gather[t.row0 + M_] / t.div) : (long)M_;
                v = t.A[arow * t.sam + (long)(k0 + K_) * t.sak];
            }
            As[K_][M_] = v;
        }
        for (int q = threadIdx.x; q < TK * TN; q += 256) {
            const int kk = q / TN, n = q % TN;
            const int kk2 = q % TK, n2 = q / TK;
            const int K_ = t.sbk == 1 ? kk2 : kk, N_ = t.sbk == 1 ? n2 : n;
            Bs[K_][N_] = (N_ < t.Nt && k0 + K_ < t.Kt) ? t.B[(long)(k0 + K_) * t.sbk + N_ * t.sbn] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < TK; ++kk) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = ty * 4 + i;
        if (m >= t.Mt) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = tx * 4 + j;
            if (n >= t.Nt) continue;
            const size_t o = (size_t)(t.scatter ? t.scatter[t.row0 + m] : m) * t.ldc + n;
            float v = acc[i][j];
            if (t.bias) v += t.bias[n];
            switch (g.kind) {
                case kRowsNN_GeLU: t.C[o] = v; t.C2[o] = gelu_f(v); break;
                case kRowsNT_dGeLU: t.C[o] = v * gelu_grad_f(t.Z[o]); break;
                case kColsT: t.C[o] = g.accumulate ? t.C[o] + v : v; break;
                default: t.C[o] = v; break;
            }
        }
    }
}
}  // namespace

void launch_ggemm_f32(const GemmArgs& a, hipStream_t st)
{
    if (a.kind == kColsT) {
        const dim3 grid((a.Nout + TN - 1) / TN, (a.K + TM - 1) / TM, a.E);
        hipLaunchKernelGGL(ggemm_f32_kernel, grid, dim3(256), 0, st, a, 0);
    } else {
        const long max_tiles = a.M / TM + a.E;   // sum_e ceil(c_e / TM) <= floor(M / TM) + E
        const int ntn = (a.Nout + TN - 1) / TN;
        hipLaunchKernelGGL(ggemm_f32_kernel, dim3((unsigned)(max_tiles * ntn)), dim3(256), 0, st, a, ntn);
    }
}

}  // namespace moe
