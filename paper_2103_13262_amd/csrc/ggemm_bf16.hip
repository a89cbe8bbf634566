// Grouped matrix products in bf16 on the CDNA4 matrix cores, fp32 accumulation: the experts'
// two fully-connected layers applied to their contiguous, variable-sized batches in ONE launch
// (Section 3.1, the dedicated linear module that runs the experts in parallel; Section 4, batching
// all samples of an expert), and the matching data- and weight-gradient products.
//
// Tile: 128 x 128 outputs per 256-thread workgroup, reduction in steps of 64 through two LDS
// stages.  Wavefronts form a 2 x 2 grid; each owns 64 x 64 outputs = 2 x 2 accumulators of
// v_mfma_f32_32x32x16_bf16.  Both operands sit in LDS as [row][k] with k contiguous (row pitch 72
// elements, so the 16-byte operand reads of 8 consecutive lanes cover all banks).  Operands whose
// memory layout has the reduction index as the slow one (weights in the forward products, both
// operands of the weight gradients) are transposed in registers on their way into LDS.
//
// Instead of the paper's per-expert library calls on several streams, the tile -> (expert, row
// block, column block) map is computed in the kernel from a prefix table the plan step wrote, and
// workgroup ids are remapped so that each XCD (own L2) works on a contiguous range of tiles.
#include "common.h"

namespace moe {

namespace {
constexpr int BM = 128, BN = 128, BK = 64;
constexpr int LDP = BK + 8;                        // LDS row pitch in elements
constexpr int STAGE_ELEMS = (BM + BN) * LDP;       // one stage: A tile then B tile
constexpr int SMEM_BYTES = 2 * STAGE_ELEMS * 2;

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef unsigned short u16;

// Global -> register -> LDS staging of one 128 x 64 operand tile.
//   TRANS == false: source is [row][k], k contiguous, pitch ld.   Each thread moves 4 x 16 B.
//   TRANS == true : source is [k][row], row contiguous, pitch ld. Each thread owns a 4(k) x 8(row)
//                   block and writes it transposed (8 x 8 B).
template <bool TRANS> struct Stager {
    uint4 r[4];
    __device__ __forceinline__ void load(const u16* __restrict__ src, long ld, int k0, int rows, int Kt)
    {
        const int tid = threadIdx.x;
        if constexpr (!TRANS) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int q = tid + 256 * i;
                const int row = q >> 3, kc = (q & 7) * 8;
                r[i] = (row < rows && k0 + kc < Kt) ? *(const uint4*)(src + (long)row * ld + k0 + kc)
                                                    : make_uint4(0, 0, 0, 0);
            }
        } else {
            const int lane = tid & 63, wave = tid >> 6;
            const int kb = lane & 15, nb = (lane >> 4) + 4 * wave;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int kr = k0 + 4 * kb + i;
                r[i] = (kr < Kt && 8 * nb < rows) ? *(const uint4*)(src + (long)kr * ld + 8 * nb)
                                                  : make_uint4(0, 0, 0, 0);
            }
        }
    }
    __device__ __forceinline__ void store(u16* __restrict__ tile) const
    {
        const int tid = threadIdx.x;
        if constexpr (!TRANS) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int q = tid + 256 * i;
                const int row = q >> 3, kc = (q & 7) * 8;
                *(uint4*)(tile + row * LDP + kc) = r[i];
            }
        } else {
            const int lane = tid & 63, wave = tid >> 6;
            const int kb = lane & 15, nb = (lane >> 4) + 4 * wave;
            const unsigned w[4][4] = {{r[0].x, r[0].y, r[0].z, r[0].w},
                                      {r[1].x, r[1].y, r[1].z, r[1].w},
                                      {r[2].x, r[2].y, r[2].z, r[2].w},
                                      {r[3].x, r[3].y, r[3].z, r[3].w}};
#pragma unroll
            for (int nn = 0; nn < 8; ++nn) {
                const int wd = nn >> 1;
                uint2 o;
                if (nn & 1) {
                    o.x = (w[0][wd] >> 16) | (w[1][wd] & 0xffff0000u);
                    o.y = (w[2][wd] >> 16) | (w[3][wd] & 0xffff0000u);
                } else {
                    o.x = (w[0][wd] & 0xffffu) | (w[1][wd] << 16);
                    o.y = (w[2][wd] & 0xffffu) | (w[3][wd] << 16);
                }
                *(uint2*)(tile + (8 * nb + nn) * LDP + 4 * kb) = o;
            }
        }
    }
};

template <int KIND>
__global__ __launch_bounds__(256) void ggemm_bf16_kernel(GemmArgs g, int ntm, int ntn)
{
    constexpr bool A_TRANS = KIND == kColsT;
    constexpr bool B_TRANS = KIND == kRowsNN || KIND == kRowsNN_GeLU || KIND == kColsT;
    extern __shared__ __align__(16) u16 smem[];

    const u16* A;  long lda;
    const u16* B;  long ldb;
    size_t c_off;  // element offset of the tile's first output
    int Mt, Nt, Kt;

    if constexpr (KIND == kColsT) {
        // C[e] (K1 x K2) = A[seg]^T B[seg]; ntm x ntn tiles per expert, experts in descending-count order.
        const int tpe = ntm * ntn;
        int ord, q;
        if ((tpe & 7) == 0) {            // each XCD takes a contiguous eighth of an expert's tiles
            const int per = tpe >> 3, xcd = blockIdx.x & 7, s = blockIdx.x >> 3;
            ord = s / per;
            q = xcd * per + (s - ord * per);
        } else {
            ord = blockIdx.x / tpe;
            q = blockIdx.x - ord * tpe;
        }
        const int e = g.order[ord];
        const int m0 = (q / ntn) * BM, n0 = (q % ntn) * BN;
        const long off = g.offsets[e];
        A = (const u16*)g.A + off * g.K + m0;     lda = g.K;
        B = (const u16*)g.B + off * g.Nout + n0;  ldb = g.Nout;
        c_off = ((size_t)e * g.K + m0) * g.Nout + n0;
        Mt = min(BM, g.K - m0);  Nt = min(BN, g.Nout - n0);  Kt = g.counts[e];
    } else {
        const int32_t* P = g.tileP + tile_height_index(BM) * (g.E + 1);
        const long T = (long)P[g.E] * ntn;
        const long chunk = (T + 7) >> 3;
        const long slot = blockIdx.x >> 3;
        const long L = (long)(blockIdx.x & 7) * chunk + slot;
        if (slot >= chunk || L >= T) return;
        int lo = 0, hi = g.E;            // largest e with P[e] * ntn <= L
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if ((long)P[mid] * ntn <= L) lo = mid; else hi = mid;
        }
        const int e = lo;
        const int mte = P[e + 1] - P[e];
        const int local = (int)(L - (long)P[e] * ntn);
        const int nt = local / mte, mt = local - nt * mte;   // row blocks fastest: neighbours share the weight panel
        const long r0 = (long)g.offsets[e] + (long)mt * BM;
        const int n0 = nt * BN;
        A = (const u16*)g.A + r0 * g.K;  lda = g.K;
        const u16* Be = (const u16*)g.B + (size_t)e * g.K * g.Nout;
        if constexpr (B_TRANS) { B = Be + n0; ldb = g.Nout; }
        else                   { B = Be + (size_t)n0 * g.K; ldb = g.K; }
        c_off = (size_t)r0 * g.Nout + n0;
        Mt = min(BM, g.counts[e] - mt * BM);  Nt = min(BN, g.Nout - n0);  Kt = g.K;
    }

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    Stager<A_TRANS> sa;
    Stager<B_TRANS> sb;
    const int nk = (Kt + BK - 1) / BK;
    if (nk > 0) {
        sa.load(A, lda, 0, Mt, Kt);
        sb.load(B, ldb, 0, Nt, Kt);
        sa.store(smem);
        sb.store(smem + BM * LDP);
    }
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const u16* tA = smem + (kt & 1) * STAGE_ELEMS;
        const u16* tB = tA + BM * LDP;
        const bool more = kt + 1 < nk;
        if (more) {
            sa.load(A, lda, (kt + 1) * BK, Mt, Kt);
            sb.load(B, ldb, (kt + 1) * BK, Nt, Kt);
        }
        const int arow = wm * 64 + (lane & 31), brow = wn * 64 + (lane & 31), koff = (lane >> 5) * 8;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8 a[2], b[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) a[i] = *(const bf16x8*)(tA + (arow + i * 32) * LDP + ks * 16 + koff);
#pragma unroll
            for (int j = 0; j < 2; ++j) b[j] = *(const bf16x8*)(tB + (brow + j * 32) * LDP + ks * 16 + koff);
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
        }
        if (more) {
            u16* nA = smem + ((kt + 1) & 1) * STAGE_ELEMS;
            sa.store(nA);
            sb.store(nA + BM * LDP);
        }
        __syncthreads();
    }

    // Accumulator element v of lane l: row (v/4)*8 + (l/32)*4 + v%4, column l%32 of its 32x32 block.
    const int ldc = g.Nout;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int col = wn * 64 + j * 32 + (lane & 31);
            if (col >= Nt) continue;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = wm * 64 + i * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
                if (row >= Mt) continue;
                const size_t o = c_off + (size_t)row * ldc + col;
                const float x = acc[i][j][v];
                if constexpr (KIND == kRowsNN_GeLU) {
                    ((u16*)g.C)[o] = f32_to_bf16(x);
                    ((u16*)g.C2)[o] = f32_to_bf16(gelu_f(x));
                } else if constexpr (KIND == kRowsNT_dGeLU) {
                    ((u16*)g.C)[o] = f32_to_bf16(x * gelu_grad_f(bf16_to_f32(((const u16*)g.Zin)[o])));
                } else if constexpr (KIND == kColsT) {
                    if (g.out_f32) {
                        float* C = (float*)g.C;
                        C[o] = g.accumulate ? C[o] + x : x;
                    } else {
                        u16* C = (u16*)g.C;
                        C[o] = f32_to_bf16(g.accumulate ? bf16_to_f32(C[o]) + x : x);
                    }
                } else {
                    ((u16*)g.C)[o] = f32_to_bf16(x);
                }
            }
        }
}

template <int KIND> void launch_kind(const GemmArgs& a, hipStream_t st)
{
    static bool attr_set = false;   // the tile needs more LDS than the default dynamic limit
    if (!attr_set) {
        if (hipFuncSetAttribute((const void*)ggemm_bf16_kernel<KIND>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                SMEM_BYTES) != hipSuccess)
            return;   // the launch below is skipped; the caller's hipGetLastError() reports the failure
        attr_set = true;
    }
    if (KIND == kColsT) {
        const int ntm = (a.K + BM - 1) / BM, ntn = (a.Nout + BN - 1) / BN;
        const long blocks = (long)a.E * ntm * ntn;
        hipLaunchKernelGGL(ggemm_bf16_kernel<KIND>, dim3((unsigned)blocks), dim3(256), SMEM_BYTES, st, a, ntm, ntn);
    } else {
        const int ntn = (a.Nout + BN - 1) / BN;
        const long max_tiles = (a.M / BM + a.E) * ntn;   // sum_e ceil(c_e / BM) <= floor(M / BM) + E
        const long blocks = (max_tiles + 7) / 8 * 8;
        hipLaunchKernelGGL(ggemm_bf16_kernel<KIND>, dim3((unsigned)blocks), dim3(256), SMEM_BYTES, st, a, 0, ntn);
    }
}
}  // namespace

void launch_ggemm_bf16(const GemmArgs& a, hipStream_t st)
{
    switch (a.kind) {
        case kRowsNN_GeLU: launch_kind<kRowsNN_GeLU>(a, st); break;
        case kRowsNN: launch_kind<kRowsNN>(a, st); break;
        case kRowsNT_dGeLU: launch_kind<kRowsNT_dGeLU>(a, st); break;
        case kRowsNT: launch_kind<kRowsNT>(a, st); break;
        default: launch_kind<kColsT>(a, st); break;
    }
}

}  // namespace moe
