// Grouped bf16 matrix products, second generation: tiles are brought from global memory straight
// into LDS (global_load_lds_dwordx4, no register staging) through a ring of STAGES buffers, so
// several reduction steps of loads are in flight while the matrix cores work on the current one.
//
// Workgroup: WM x WN wavefronts, each owning TM x TN accumulators of v_mfma_f32_32x32x16_bf16
// (wave tile 32*TM x 32*TN, workgroup tile BM x BN), reduction step 32.
//
// LDS layouts (each wave-level load instruction fills one contiguous 1 KB piece, lane p -> byte
// 16*p, so a layout is chosen by choosing which global 16-byte chunk each lane fetches):
//   k-contiguous source ([row][k]):  LDS row = 64 B = 4 chunks; chunk c of row r sits at position
//       c ^ swz(r), swz(r) = ((r>>1)&3) ^ ((r>>3)&1); operand reads are ds_read_b128 and are free
//       of bank conflicts for 8- and for 16-lane groups.
//   row-contiguous source ([k][row], the reduction index is the slow one: weights in the forward
//       products, both operands of the weight gradients): LDS keeps the global layout, k-row =
//       BM/8 chunks, chunk c of k-row k at position c ^ 2*(k&3); operands are gathered with
//       ds_read_b64_tr_b16, which hands lane i of a 16-lane group column i of a 4(k) x 16 block.
//
// Rows / columns outside the tile's valid extent are fetched from a clamped (valid) address and
// their results are never stored.  Reduction rows past the end of an expert's segment (weight
// gradients only) are fetched from a page of zeros.
#include <cstdio>
#include <cstdlib>
#include <type_traits>
#include <utility>
#include <vector>

#include "common.h"

namespace moe {
namespace dma {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef unsigned short u16;
#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))
#define GLB_PTR(p) ((const __attribute__((address_space(1))) void*)(p))

// Chunk swizzle of k-contiguous tiles (row r, 16-byte chunk c sits at position c ^ swz(r)).
//   BK = 32: 4 chunks per row;  BK = 64: 8 chunks per row.
template <int BK> __device__ __forceinline__ int swz(int r)
{
    if constexpr (BK == 32) return ((r >> 1) & 3) ^ ((r >> 3) & 1);
    else return (r >> 1) & 7;
}

// s_waitcnt vmcnt(N) only (export and LDS counters left at their maxima), gfx9 encoding.
template <int N> __device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt range");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}
template <int PER, int MAXG> __device__ __forceinline__ void wait_groups(int groups)
{   // allow `groups` (0..MAXG) load groups of PER instructions each to stay in flight
    if constexpr (MAXG == 0) { wait_vmcnt<0>(); }
    else {
        if (groups >= MAXG) wait_vmcnt<PER * MAXG>();
        else wait_groups<PER, MAXG - 1>(groups);
    }
}

template <int KIND, int WM, int WN, int TM, int TN, int STAGES, int BK_>
struct Cfg {
    static constexpr int BK = BK_;
    static constexpr int NW = WM * WN, NT = NW * 64;
    static constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
    static constexpr bool A_TRANS = KIND == kColsT;
    static constexpr bool B_TRANS = KIND == kRowsNN || KIND == kRowsNN_GeLU || KIND == kColsT;
    static constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2, STAGE_BYTES = A_BYTES + B_BYTES;
    static constexpr int LA = A_BYTES / 1024 / NW, LB = B_BYTES / 1024 / NW;   // wave-level loads per wave and stage
    static constexpr int SMEM = STAGES * STAGE_BYTES;
    static_assert(A_BYTES % (1024 * NW) == 0 && B_BYTES % (1024 * NW) == 0, "tile must split evenly over waves");
};

// Per-lane source pointers of one operand for reduction block 0 (advanced by the caller) and the
// reduction offset inside a block that the lane's chunk starts at (krow).
//   !TRANS: src[row][k]; lane p of load j covers row j*16 + p/4, logical chunk (p&3) ^ swz(p/4).
//    TRANS: src[k][row]; CPR = R/8 chunks per k-row; lane p of load j covers k-row j*(64/CPR) + p/CPR,
//           logical chunk (p % CPR) ^ 2*(krow & 3).
template <bool TRANS, int R, int NW, int L, int BK>
__device__ __forceinline__ void setup_ptrs(const u16* base, long ld, int valid, int wave, int lane, const u16* (&ptr)[L],
                                           int (&krow)[L])
{
#pragma unroll
    for (int i = 0; i < L; ++i) {
        const int j = wave + i * NW;
        if constexpr (!TRANS) {
            constexpr int CK = BK / 8;                      // chunks per row; one load covers 64 / CK rows
            int row = j * (64 / CK) + lane / CK;
            const int c = (lane % CK) ^ swz<BK>(row);
            row = row < valid ? row : valid - 1;
            ptr[i] = base + (long)row * ld + c * 8;
            krow[i] = c * 8;            // reduction offset of this lane's chunk inside a block
        } else {
            constexpr int CPR = R / 8;
            const int kr = j * (64 / CPR) + lane / CPR;
            int c = (lane % CPR) ^ (2 * (kr & 3));
            c = c * 8 < valid ? c : 0;
            ptr[i] = base + (long)kr * ld + c * 8;
            krow[i] = kr;
        }
    }
}

template <int KIND, int WM, int WN, int TM, int TN, int STAGES, int BK, int OCC>
__global__ __launch_bounds__(WM * WN * 64, OCC) void ggemm_dma_kernel(GemmArgs g, int ntm, int ntn)
{
    using C = Cfg<KIND, WM, WN, TM, TN, STAGES, BK>;
    constexpr int BM = C::BM, BN = C::BN;
    extern __shared__ __align__(1024) char smem[];
    long long ts[6];
    ts[0] = wall_clock64();

    const u16* A;  long lda;
    const u16* B;  long ldb;
    size_t c_off;
    int Mt, Nt, Kt;
    if constexpr (KIND == kColsT) {
        const int tpe = ntm * ntn;
        int ord, q;
        if ((tpe & 7) == 0) {
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
        int lo = 0, hi = g.E;
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if ((long)P[mid] * ntn <= L) lo = mid; else hi = mid;
        }
        const int e = lo;
        const int mte = P[e + 1] - P[e];
        const int local = (int)(L - (long)P[e] * ntn);
        // Order inside an expert: groups of up to GM row blocks; inside a group the row block runs fastest,
        // then the column block.  Tiles that run at the same time on one XCD then form a patch that shares
        // both the activation panels (across its column blocks) and the weight panels (across its row blocks).
        constexpr int GM = 8;
        int nt, mt;
        {
            const int full = mte / GM, per_group = GM * ntn;
            const int gi = local / per_group;
            if (gi < full) {
                const int r = local - gi * per_group;
                nt = r / GM;
                mt = gi * GM + (r - nt * GM);
            } else {
                const int rem = mte - full * GM;
                const int r = local - full * per_group;
                nt = r / rem;
                mt = full * GM + (r - nt * rem);
            }
        }
        const long r0 = (long)g.offsets[e] + (long)mt * BM;
        const int n0 = nt * BN;
        A = (const u16*)g.A + r0 * g.K;  lda = g.K;
        const u16* Be = (const u16*)g.B + (size_t)e * g.K * g.Nout;
        if constexpr (C::B_TRANS) { B = Be + n0; ldb = g.Nout; }
        else                      { B = Be + (size_t)n0 * g.K; ldb = g.K; }
        c_off = (size_t)r0 * g.Nout + n0;
        Mt = min(BM, g.counts[e] - mt * BM);  Nt = min(BN, g.Nout - n0);  Kt = g.K;
    }

    ts[1] = wall_clock64();
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform, kept in a scalar register
    const int wm = wave / WN, wn = wave % WN;
    const int nk = (Kt + BK - 1) / BK;

    // ---- global -> LDS streams ----
    const u16* pa[C::LA]; int ka[C::LA];
    const u16* pb[C::LB]; int kb[C::LB];
    setup_ptrs<C::A_TRANS, BM, C::NW, C::LA, BK>(A, lda, Mt, wave, lane, pa, ka);
    setup_ptrs<C::B_TRANS, BN, C::NW, C::LB, BK>(B, ldb, Nt, wave, lane, pb, kb);
    const long stepA = C::A_TRANS ? (long)BK * lda : BK, stepB = C::B_TRANS ? (long)BK * ldb : BK;
    const u16* zeros = (const u16*)g.zeros + lane * 8;
    // reduction indices past Kt are read from the zero page: always possible for the weight gradients (Kt = rows
    // of the expert), and for the other kinds only when a block is deeper than the 32 that divides every width
    constexpr bool KMASK = KIND == kColsT || BK > 32;

    // The loads are written as inline assembly so that the compiler does not serialise them against
    // the LDS reads of other ring slots (it cannot tell the slots apart and would wait for all loads
    // before every read); the ordering is enforced by the explicit vmcnt waits and barriers below.
    const unsigned lds_base = (unsigned)(uintptr_t)LDS_PTR(char, smem);
    // One wave-level load (index l of the LA + LB loads this wave owns per block) of reduction block kt
    // into ring slot kt % STAGES.  l is a compile-time constant at every call site.
    auto issue_one = [&](int kt, auto lc) {
        constexpr int l = decltype(lc)::value;
        const unsigned sA = lds_base + (kt % STAGES) * C::STAGE_BYTES + wave * 1024;
        if constexpr (l < C::LA) {
            const u16* src = pa[l];
            if constexpr (KMASK) src = (kt * BK + ka[l] < Kt) ? src : zeros;
            asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off"
                         :: "s"(sA + l * C::NW * 1024), "v"(src) : "memory");
            pa[l] += stepA;
        } else {
            constexpr int i = l - C::LA;
            const u16* src = pb[i];
            if constexpr (KMASK) src = (kt * BK + kb[i] < Kt) ? src : zeros;
            asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off"
                         :: "s"(sA + C::A_BYTES + i * C::NW * 1024), "v"(src) : "memory");
            pb[i] += stepB;
        }
    };
    auto issue = [&](int kt) {   // all loads of block kt at once (prologue)
        [&]<int... L>(std::integer_sequence<int, L...>) {
            (issue_one(kt, std::integral_constant<int, L>{}), ...);
        }(std::make_integer_sequence<int, C::LA + C::LB>{});
    };
    // ---- per-lane LDS offsets of the MFMA operand fetches (within one operand tile, ks = 0) ----
    int offA[TM], offB[TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int rb = (wm * TM + i) * 32;
        if constexpr (!C::A_TRANS) {
            offA[i] = (rb + (lane & 31)) * (BK * 2) + ((((lane >> 5)) ^ swz<BK>(lane & 31)) << 4);
        } else {
            const int s = lane & 15, col = rb + ((lane >> 4) & 1) * 16 + 4 * (s & 3);
            offA[i] = ((lane >> 5) * 8 + (s >> 2)) * (BM * 2) + ((((col >> 3)) ^ (2 * (s >> 2))) << 4) + (col & 7) * 2;
        }
    }
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int rb = (wn * TN + j) * 32;
        if constexpr (!C::B_TRANS) {
            offB[j] = (rb + (lane & 31)) * (BK * 2) + ((((lane >> 5)) ^ swz<BK>(lane & 31)) << 4);
        } else {
            const int s = lane & 15, col = rb + ((lane >> 4) & 1) * 16 + 4 * (s & 3);
            offB[j] = ((lane >> 5) * 8 + (s >> 2)) * (BN * 2) + ((((col >> 3)) ^ (2 * (s >> 2))) << 4) + (col & 7) * 2;
        }
    }
    auto fetchA = [&](const char* tile, int i, int ks) -> bf16x8 {
        if constexpr (!C::A_TRANS) {
            return *(const bf16x8*)(tile + (offA[i] ^ (ks << 5)));
        } else {
            const char* p = tile + offA[i] + ks * 16 * (BM * 2);
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, p));
            const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, p + 4 * (BM * 2)));
            const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            return __builtin_bit_cast(bf16x8, v);
        }
    };
    auto fetchB = [&](const char* tile, int j, int ks) -> bf16x8 {
        if constexpr (!C::B_TRANS) {
            return *(const bf16x8*)(tile + (offB[j] ^ (ks << 5)));
        } else {
            const char* p = tile + offB[j] + ks * 16 * (BN * 2);
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, p));
            const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, p + 4 * (BN * 2)));
            const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            return __builtin_bit_cast(bf16x8, v);
        }
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // row blocks of this wave that hold at least one valid row (tail tiles skip the rest)
    int tm_act = (Mt - wm * TM * 32 + 31) / 32;
    tm_act = tm_act < 0 ? 0 : (tm_act > TM ? TM : tm_act);

    // Software pipeline.  Ring slot kt % STAGES holds reduction block kt.  The operand registers are
    // double-buffered: while the matrix cores work on one 16-deep step, the LDS reads of the next step
    // (which may belong to the next block) are in flight.  Per block there is one barrier, placed after
    // this wave's last LDS read of the block, so that the slot can be refilled right behind it.
    auto main_loop = [&](auto full_tag) {
        constexpr bool FULL = decltype(full_tag)::value;
        constexpr int PER = C::LA + C::LB;
        static_assert((BK / 16) % 2 == 0, "even number of MFMA steps per block");
        constexpr int KS = BK / 16;                         // 16-deep MFMA steps per block (even)
        bf16x8 fa[2][TM], fb[2][TN];                        // operand registers, double-buffered by step parity
        auto fetch = [&](int slot, int ks, bf16x8 (&a)[TM], bf16x8 (&b)[TN]) {
            const char* tA = smem + slot * C::STAGE_BYTES;
            const char* tB = tA + C::A_BYTES;
#pragma unroll
            for (int j = 0; j < TN; ++j) b[j] = fetchB(tB, j, ks);
#pragma unroll
            for (int i = 0; i < TM; ++i)
                if (FULL || i < tm_act) a[i] = fetchA(tA, i, ks);
        };
        // One 16-deep MFMA step.  The loads of the block that refills the slot freed at the last barrier
        // are spread over the KS steps that follow that barrier (SLOTS = KS * TM places, one before each
        // accumulator row), so that they do not hold up the matrix cores in one burst.
        constexpr int SLOTS = KS * TM;
        auto mma = [&](const bf16x8 (&a)[TM], const bf16x8 (&b)[TN], auto step_c, int load_kt) {
            constexpr int STEP = decltype(step_c)::value;
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                if (load_kt >= 0) {
                    [&]<int... L>(std::integer_sequence<int, L...>) {
                        ((L * SLOTS / PER == STEP * TM + i ? (issue_one(load_kt, std::integral_constant<int, L>{}), 0) : 0), ...);
                    }(std::make_integer_sequence<int, PER>{});
                }
                if (FULL || i < tm_act) {
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
                }
            }
        };
        if (nk == 0) return;
#pragma unroll
        for (int s = 0; s < STAGES; ++s)
            if (s < nk) issue(s);
        wait_groups<PER, STAGES - 1>(min(nk - 1, STAGES - 1));   // block 0 has landed
        __builtin_amdgcn_s_barrier();
        ts[2] = wall_clock64();
        fetch(0, 0, fa[0], fb[0]);
        int load_kt = -1;   // block being loaded piecewise (into the slot freed at the last barrier), or -1
        auto steps_before_barrier = [&](int slot) {   // steps 0 .. KS-2 of a block: load pieces 1 .. KS-1
            [&]<int... S>(std::integer_sequence<int, S...>) {
                ((fetch(slot, S + 1, fa[(S + 1) & 1], fb[(S + 1) & 1]),
                  mma(fa[S & 1], fb[S & 1], std::integral_constant<int, S + 1>{}, load_kt)), ...);
            }(std::make_integer_sequence<int, KS - 1>{});
        };
        for (int kt = 0; kt + 1 < nk; ++kt) {
            steps_before_barrier(kt % STAGES);
            // own loads of block kt+1 have landed (blocks kt+2 .. may stay in flight) and own LDS
            // reads of block kt are complete; after the barrier that holds for every wave
            wait_groups<PER, STAGES - 2>(min(nk - 2 - kt, STAGES - 2));
            __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0), other counters untouched
            __builtin_amdgcn_s_barrier();
            load_kt = kt + STAGES < nk ? kt + STAGES : -1;
            fetch((kt + 1) % STAGES, 0, fa[0], fb[0]);
            mma(fa[1], fb[1], std::integral_constant<int, 0>{}, load_kt);
        }
        steps_before_barrier((nk - 1) % STAGES);   // last block: load_kt is -1 here, nothing left to prefetch
        mma(fa[1], fb[1], std::integral_constant<int, 0>{}, -1);
    };
    if (tm_act == TM) main_loop(std::true_type{});
    else main_loop(std::false_type{});   // tail tiles skip the 32-row blocks that hold no valid row

    // ---- epilogue ----
    // Accumulator element v of lane l is row (v/4)*8 + (l/32)*4 + v%4, column l%32 of its 32x32 block.
    // Each wave passes one 32-row block at a time through a private fp32 LDS patch and reads it back
    // row-wise, 8 consecutive columns per lane, so that global memory sees 16-byte pieces of whole rows.
    constexpr int PITCH = TN * 32 + 4;                       // floats; rows 4 apart land in different banks
    static_assert(C::NW * 32 * PITCH * 4 <= C::SMEM, "epilogue patch must fit in the ring");
    __syncthreads();                                         // all waves are done with the ring
    ts[3] = wall_clock64();
    float* patch = (float*)smem + wave * (32 * PITCH);
    constexpr int CPRW = TN * 4;                             // 8-column pieces per row of the wave tile
    const int ldc = g.Nout;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        if (i >= tm_act) break;
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v)
                patch[((v >> 2) * 8 + (lane >> 5) * 4 + (v & 3)) * PITCH + j * 32 + (lane & 31)] = acc[i][j][v];
        // (same wave wrote and reads: LDS operations of one wave complete in order)
        for (int q = lane; q < 32 * CPRW; q += 64) {
            const int r = q / CPRW, cp = q % CPRW;
            const int row = (wm * TM + i) * 32 + r, col = wn * TN * 32 + cp * 8;
            if (row >= Mt || col >= Nt) continue;
            const float4 lo = *(const float4*)(patch + r * PITCH + cp * 8);
            const float4 hi = *(const float4*)(patch + r * PITCH + cp * 8 + 4);
            float x[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
            const size_t o = c_off + (size_t)row * ldc + col;
            auto pack = [](const float* f) {
                return make_uint4(pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]), pack_bf16x2(f[4], f[5]),
                                  pack_bf16x2(f[6], f[7]));
            };
            auto unpack = [](const uint4 u, float* f) {
                const unsigned w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    f[2 * t] = __uint_as_float(w[t] << 16);
                    f[2 * t + 1] = __uint_as_float(w[t] & 0xffff0000u);
                }
            };
            if constexpr (KIND == kRowsNN_GeLU) {
                *(uint4*)((u16*)g.C + o) = pack(x);
#pragma unroll
                for (int t = 0; t < 8; ++t) x[t] = gelu_fast(x[t]);
                *(uint4*)((u16*)g.C2 + o) = pack(x);
            } else if constexpr (KIND == kRowsNT_dGeLU) {
                float z[8];
                unpack(*(const uint4*)((const u16*)g.Zin + o), z);
#pragma unroll
                for (int t = 0; t < 8; ++t) x[t] *= gelu_grad_fast(z[t]);
                *(uint4*)((u16*)g.C + o) = pack(x);
            } else if constexpr (KIND == kColsT) {
                if (g.out_f32) {
                    float4* Cf = (float4*)((float*)g.C + o);
                    if (g.accumulate) {
                        const float4 p0 = Cf[0], p1 = Cf[1];
                        x[0] += p0.x; x[1] += p0.y; x[2] += p0.z; x[3] += p0.w;
                        x[4] += p1.x; x[5] += p1.y; x[6] += p1.z; x[7] += p1.w;
                    }
                    Cf[0] = make_float4(x[0], x[1], x[2], x[3]);
                    Cf[1] = make_float4(x[4], x[5], x[6], x[7]);
                } else {
                    uint4* Ch = (uint4*)((u16*)g.C + o);
                    if (g.accumulate) {
                        float p[8];
                        unpack(*Ch, p);
#pragma unroll
                        for (int t = 0; t < 8; ++t) x[t] += p[t];
                    }
                    *Ch = pack(x);
                }
            } else {
                *(uint4*)((u16*)g.C + o) = pack(x);
            }
        }
    }
    if (g.trace && threadIdx.x == 0) {
        ts[4] = wall_clock64();
        long long* t = g.trace + (size_t)blockIdx.x * 8;
        t[0] = ts[0]; t[1] = ts[1]; t[2] = ts[2]; t[3] = ts[3]; t[4] = ts[4]; t[5] = nk; t[6] = tm_act; t[7] = 1;
    }
}

template <int KIND, int WM, int WN, int TM, int TN, int STAGES, int BK, int OCC = 1>
void launch_cfg(const GemmArgs& a, hipStream_t st)
{
    using C = Cfg<KIND, WM, WN, TM, TN, STAGES, BK>;
    auto kern = ggemm_dma_kernel<KIND, WM, WN, TM, TN, STAGES, BK, OCC>;
    static bool attr_set = false;   // the LDS ring is larger than the default dynamic limit
    if (!attr_set) {
        if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, C::SMEM) != hipSuccess)
            return;   // launch skipped; the caller's hipGetLastError() reports the failure
        attr_set = true;
    }
    long blocks;
    int ntm = 0, ntn = (a.Nout + C::BN - 1) / C::BN;
    if (KIND == kColsT) {
        ntm = (a.K + C::BM - 1) / C::BM;
        blocks = (long)a.E * ntm * ntn;
    } else {
        const long max_tiles = (a.M / C::BM + a.E) * ntn;
        blocks = (max_tiles + 7) / 8 * 8;
    }
    static const bool trace_on = getenv("MOE355_TRACE") != nullptr;   // development only
    GemmArgs b = a;
    if (trace_on) {
        static long long* buf = nullptr;
        if (!buf) (void)hipMalloc(&buf, 8 * sizeof(long long) * 65536);
        b.trace = blocks <= 65536 ? buf : nullptr;
        if (b.trace) (void)hipMemsetAsync(buf, 0, 8 * sizeof(long long) * blocks, st);
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(C::NT), C::SMEM, st, b, ntm, ntn);
    if (trace_on && b.trace) {
        std::vector<long long> h(8 * blocks);
        (void)hipStreamSynchronize(st);
        (void)hipMemcpy(h.data(), b.trace, h.size() * sizeof(long long), hipMemcpyDeviceToHost);
        double ph[4] = {0, 0, 0, 0}; long n = 0, nfull = 0; long long tmin = 0, tmax = 0;
        for (long i = 0; i < blocks; ++i) {
            const long long* t = &h[8 * i];
            if (!t[7]) continue;
            if (!n || t[0] < tmin) tmin = t[0];
            if (!n || t[4] > tmax) tmax = t[4];
            ++n;
            if (t[6] != TM) continue;
            ++nfull;
            for (int k = 0; k < 4; ++k) ph[k] += (double)(t[k + 1] - t[k]);
        }
        fprintf(stderr, "[trace kind %d cfg %dx%dx%d] blocks %ld active %ld full %ld span %.1f us | per full tile (us): decode %.2f "
                "prologue %.2f mainloop %.2f epilogue %.2f\n", KIND, C::BM, C::BN, BK, blocks, n, nfull, (tmax - tmin) * 0.01,
                ph[0] / nfull * 0.01, ph[1] / nfull * 0.01, ph[2] / nfull * 0.01, ph[3] / nfull * 0.01);
    }
}

template <int KIND> void launch_kind(const GemmArgs& a, hipStream_t st)
{
    switch (0) {   // development switch between tile configurations
        case 1: launch_cfg<KIND, 2, 2, 4, 4, 2, 64>(a, st); break;   // 256x256, BK 64, 2 stages
        case 2: launch_cfg<KIND, 2, 2, 4, 2, 3, 64>(a, st); break;   // 256x128, BK 64, 3 stages
        case 3: launch_cfg<KIND, 2, 4, 4, 2, 4, 32>(a, st); break;   // 256x256, 8 waves, BK 32, 4 stages
        case 8: launch_cfg<KIND, 2, 2, 4, 4, 4, 32>(a, st); break;   // 256x256, 4 waves, BK 32, 4 stages
        case 9: launch_cfg<KIND, 2, 4, 4, 2, 5, 32>(a, st); break;   // 256x256, 8 waves, BK 32, 5 stages (160 KB)
        case 10: launch_cfg<KIND, 2, 2, 4, 4, 5, 32>(a, st); break;  // 256x256, 4 waves, BK 32, 5 stages (160 KB)
        case 11: launch_cfg<KIND, 4, 2, 2, 2, 3, 64>(a, st); break;  // 256x128, 8 waves (64x64 each), BK 64, 3 stages
        case 12: launch_cfg<KIND, 2, 4, 4, 1, 3, 64>(a, st); break;  // 256x128, 8 waves (128x32 each), BK 64, 3 stages
        case 13: launch_cfg<KIND, 2, 2, 4, 2, 3, 64>(a, st); break;  // 256x128, 4 waves (128x64 each), BK 64, 3 stages
        case 5: launch_cfg<KIND, 2, 2, 4, 2, 3, 32, 2>(a, st); break; // 256x128, 4 waves, BK 32, 3 stages, 2 workgroups per CU
        case 6: launch_cfg<KIND, 2, 2, 2, 4, 3, 32, 2>(a, st); break; // 128x256, same
        case 7: launch_cfg<KIND, 2, 2, 4, 2, 2, 32, 3>(a, st); break; // 256x128, 2 stages, 3 workgroups per CU
        default: launch_cfg<KIND, 2, 4, 4, 2, 2, 64>(a, st); break;  // 256x256, 8 waves, BK 64, 2 stages
    }
}
}  // namespace dma

void launch_ggemm_bf16_dma(const GemmArgs& a, hipStream_t st)
{
    using namespace dma;
    switch (a.kind) {
        case kRowsNN_GeLU: launch_kind<kRowsNN_GeLU>(a, st); break;
        case kRowsNN: launch_kind<kRowsNN>(a, st); break;
        case kRowsNT_dGeLU: launch_kind<kRowsNT_dGeLU>(a, st); break;
        case kRowsNT: launch_kind<kRowsNT>(a, st); break;
        default: launch_kind<kColsT>(a, st); break;
    }
}

}  // namespace moe
