// Gate linear layer, top-k and the softmax over the k selected logits for bf16 inputs and 17 to 256 experts
// (Algorithm 1: score = G(x), indices = ArgMax_k(score); the gate is one fully-connected layer, Section 5.2),
// with the selection still that of exact arithmetic.
//
// The logits of all experts are only needed to find out which few can be among the k largest; their values enter the
// result through the k selected ones.  So:
//  (1) all logits in fp32 on the bf16 matrix cores (products of two bf16 values are exact in fp32; only the summation
//      rounds), together with the same product of the absolute values, S[t,e] = sum_i |x_i| |w_ie| + |b_e|, which
//      bounds the rounding error of a sum of d + 1 terms in ANY order by (d + 1) 2^-24 S (the kernel takes four
//      times that, and for S the largest value among the workgroup's tokens and experts);
//  (2) per token the k-th largest fp32 logit v_k (k rounds of a wavefront-wide argmax, four tokens interleaved);
//      an expert can only be among the exact k largest if its fp32 logit is at least v_k minus twice the bound: these
//      CANDIDATES are usually just the k largest, sometimes one or two more (near-ties, equal gate columns);
//  (3) the candidates' logits again in fp64 (16 lanes per token and candidate, each a slice of the features, one fixed
//      butterfly: equal gate columns give equal sums), the k largest with ties to the lower expert id are the
//      selection, their softmax the scores;
//  (4) a token with more than 16 candidates (e.g. an all-zero row: every logit equal), or of a workgroup whose S is not
//      finite, goes on a list for a second kernel that evaluates all E logits in fp64.
//
// Kernels: gate_prep (transposed gate matrix [E][d], so that an expert's weights are contiguous; clears the list's
// counter), gate_bf16_kernel<G> (32 tokens per workgroup of 8 wavefronts, G = 64, 128 or 256 expert columns; a
// wavefront takes 32 columns and, where G < 256, a share of every slab's reduction steps; both operands staged
// through LDS in 64-feature slabs, swizzled for conflict-free 16-byte reads), gate_fix_kernel (a wavefront per listed
// token).
#include "common.h"

namespace moe {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef unsigned short u16;

constexpr int kTok = 32;            // tokens per workgroup
constexpr int kWaves = 8;           // wavefronts per workgroup
constexpr int kTokW = kTok / kWaves; // tokens whose selection a wavefront does (16 lanes each in the fp64 part)
constexpr int kSlab = 64;           // features per LDS slab (128 bytes per row)
constexpr int kCand = 16;           // candidates per token that the first kernel handles itself
constexpr float kErrFactor = 4.0f;  // safety factor on the textbook bound (d + 1) 2^-24 S of an fp32 sum in any order
constexpr int kFixWaves = 1024;     // wavefronts of the second kernel's fixed grid
constexpr int kNone = 0x7fffffff;   // "no expert": loses every tie
static_assert(kCand > kMaxK && kTokW * 16 == 64, "16 lanes per token must hold the k + 1 largest");

// LDS of gate_bf16_kernel<G>: two slabs of (32 token rows + G gate rows) x 128 bytes; after the last slab the same
// bytes hold the fp32 logits [parts][32][G + 1]; then the candidates' expert ids and the parts' largest S.
template <int G> struct Lds {
    static constexpr int kParts = kWaves / (G / 32);
    static constexpr int kSlabBytes = (kTok + G) * kSlab * 2;
    static constexpr int kLogitBytes = kParts * kTok * (G + 1) * 4;
    static constexpr int kMain = ((2 * kSlabBytes > kLogitBytes ? 2 * kSlabBytes : kLogitBytes) + 255) & ~255;
    static constexpr int kTotal = kMain + kTok * kCand * 4 + 64;
};

__device__ __forceinline__ bool better(float v, int i, float bv, int bi) { return v > bv || (v == bv && i < bi); }
__device__ __forceinline__ bool better(double v, int i, double bv, int bi) { return v > bv || (v == bv && i < bi); }

template <typename T>
__global__ __launch_bounds__(256) void gate_prep(const T* __restrict__ Wg, T* __restrict__ WgT, int d, int E, int32_t* __restrict__ fail)
{
    const long i = (long)blockIdx.x * 256 + threadIdx.x;   // index into WgT [E][d]
    if (i == 0) fail[0] = 0;
    if (i < (long)d * E) {
        const int e = (int)(i / d), f = (int)(i - (long)e * d);
        WgT[i] = Wg[(size_t)f * E + e];
    }
}

// sum_i x_i w_i in fp64 over the 16-byte pieces c = first, first + 16, ... of two rows (ascending), two gate rows at once
__device__ __forceinline__ void dot2_fp64(const u16* __restrict__ xr, const u16* __restrict__ w0, const u16* __restrict__ w1, int d,
                                          int first, double& s0, double& s1)
{
    s0 = 0.0; s1 = 0.0;
#pragma unroll 4
    for (int c = first; c < d / 8; c += 16) {
        const uint4 xv = *(const uint4*)(xr + c * 8), a = *(const uint4*)(w0 + c * 8), b = *(const uint4*)(w1 + c * 8);
        const unsigned xs[4] = {xv.x, xv.y, xv.z, xv.w}, as[4] = {a.x, a.y, a.z, a.w}, bs[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const double xl = (double)__uint_as_float(xs[q] << 16), xh = (double)__uint_as_float(xs[q] & 0xffff0000u);
            s0 = fma(xl, (double)__uint_as_float(as[q] << 16), s0);
            s0 = fma(xh, (double)__uint_as_float(as[q] & 0xffff0000u), s0);
            s1 = fma(xl, (double)__uint_as_float(bs[q] << 16), s1);
            s1 = fma(xh, (double)__uint_as_float(bs[q] & 0xffff0000u), s1);
        }
    }
}

template <int G>
__global__ __launch_bounds__(kWaves * 64) void gate_bf16_kernel(const u16* __restrict__ X, const u16* __restrict__ WgT,
                                                                const float* __restrict__ bg, int N, int d, int E, int k,
                                                                int32_t* __restrict__ topk_idx, float* __restrict__ topk_w,
                                                                int32_t* __restrict__ fail)
{
    using L = Lds<G>;
    constexpr int EB = G / 32;          // blocks of 32 expert columns
    constexpr int KP = L::kParts;       // wavefronts sharing a block: each takes every KP-th reduction step
    constexpr int WP = G / 64;          // gate pieces a thread stages per slab
    constexpr int NC = G / 64;          // logits per lane and token in the selection
    extern __shared__ __align__(1024) char smem[];
    float (*s_logit)[kTok][G + 1] = (float (*)[kTok][G + 1])smem;                 // (aliases the slabs)
    int (*s_cand)[kCand] = (int (*)[kCand])(smem + L::kMain);
    int* s_maxabs = (int*)(smem + L::kMain + kTok * kCand * 4);                   // [KP] bit patterns of the parts' largest S
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int eb = wave % EB, kp = wave / EB;
    const int t0 = blockIdx.x * kTok;
    if (tid < KP) s_maxabs[tid] = 0;
    float bias_sel[NC];                                             // the biases of experts lane + 64 c, for the selection below
#pragma unroll
    for (int c = 0; c < NC; ++c) bias_sel[c] = (bg && lane + 64 * c < E) ? bg[lane + 64 * c] : 0.f;

    // staging: thread -> 16-byte pieces of the slab.  Piece q of row r sits at r * 128 + ((q ^ swz(r)) << 4),
    // swz(r) = (r >> 1) & 7: the 32 rows that a fragment read touches then fall into all banks evenly.
    // X rows: 32 x 8 = 256 pieces (threads 0..255); gate rows: G x 8 pieces (WP per thread).
    const int srow = tid >> 3, sq = tid & 7;                       // this thread's piece inside a block of 64 rows
    auto slab_off = [](int r, int q) { return r * (kSlab * 2) + ((q ^ ((r >> 1) & 7)) << 4); };
    const u16* xsrc = X + (size_t)min(t0 + (srow & (kTok - 1)), N - 1) * d;   // (threads 256.. load what threads 0.. load and drop it)
    const u16* wsrc[WP];
#pragma unroll
    for (int u = 0; u < WP; ++u) wsrc[u] = WgT + (size_t)min(u * 64 + srow, E - 1) * d;   // rows past E: a copy of the last, never kept
    // fragments of v_mfma_f32_32x32x16_bf16: lane l holds reduction indices (l / 32) * 8 .. + 7 of row / column l % 32
    const int frow = lane & 31, fhalf = lane >> 5;
    constexpr unsigned kAbs = 0x7fff7fffu;
    const int nslab = (d + 2 * kSlab - 1) / (2 * kSlab) * 2;       // an even number of slabs; what lies past d is zero

    // The loop below has no branches on purpose: every load is issued (from a clamped address) and its value
    // replaced by zero where it lies past d, so that loads stay in flight across the barriers.
    auto fetch = [&](int s, u32x4& xv, u32x4 (&wv)[WP]) __attribute__((always_inline)) {          // slab s -> registers
        const int f = s * kSlab + sq * 8;
        const bool in = f < d;
        const int fo = in ? f : 0;
        const u32x4 zero = {0u, 0u, 0u, 0u};
        const u32x4 x = *(const u32x4*)(xsrc + fo);
        xv = in ? x : zero;
#pragma unroll
        for (int u = 0; u < WP; ++u) {
            const u32x4 w = *(const u32x4*)(wsrc[u] + fo);
            wv[u] = in ? w : zero;
        }
    };
    auto stash = [&](int buf, const u32x4& xv, const u32x4 (&wv)[WP]) __attribute__((always_inline)) {
        char* base = smem + buf * L::kSlabBytes;
        if (tid < 256) *(u32x4*)(base + slab_off(srow, sq)) = xv;
#pragma unroll
        for (int u = 0; u < WP; ++u) *(u32x4*)(base + slab_off(kTok + u * 64 + srow, sq)) = wv[u];
    };
    f32x16 acc, acc_abs;
#pragma unroll
    for (int v = 0; v < 16; ++v) { acc[v] = 0.f; acc_abs[v] = 0.f; }
    auto multiply = [&](int buf) __attribute__((always_inline)) {                                  // the slab in buffer buf into the accumulators
        const char* base = smem + buf * L::kSlabBytes;
#pragma unroll
        for (int i = 0; i < kSlab / 16 / KP; ++i) {                 // this wavefront's reduction steps kp, kp + KP, ...
            const int q = 2 * (kp + KP * i) + fhalf;
            const u32x4 a = *(const u32x4*)(base + slab_off(frow, q));
            const u32x4 b = *(const u32x4*)(base + slab_off(kTok + eb * 32 + frow, q));
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
            acc_abs = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a & kAbs), __builtin_bit_cast(bf16x8, b & kAbs),
                                                              acc_abs, 0, 0, 0);
        }
    };
    {
        // two slabs are on their way in registers while one is multiplied: slab s waits in buffer s & 1, slab s + 1 is
        // written there once everyone is past slab s - 1 (the barrier before slab s is multiplied)
        u32x4 xa, wa[WP], xb, wb[WP];
        fetch(0, xa, wa);
        fetch(1, xb, wb);
        stash(0, xa, wa);
        for (int s = 0; s < nslab; s += 2) {
            fetch(s + 2, xa, wa);
            __syncthreads();
            multiply(0);
            stash(1, xb, wb);
            fetch(s + 3, xb, wb);
            __syncthreads();
            multiply(1);
            stash(0, xa, wa);
        }
    }
    __syncthreads();                                                // the slabs are done with: their bytes now take the logits
    // accumulator element v of lane l: row (v / 4) * 8 + (l / 32) * 4 + v % 4, column l % 32
    {
        const int col = eb * 32 + frow;
        float sa_max = 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = (v >> 2) * 8 + fhalf * 4 + (v & 3);
            s_logit[kp][row][col] = acc[v];
            float sa = acc_abs[v];
            if (!(sa < INFINITY)) sa = INFINITY;                    // (NaN or overflow: nothing can be bounded)
            sa_max = fmaxf(sa_max, col < E ? sa : 0.f);
        }
        if (kp == 0 && bg && col < E) sa_max += fabsf(bg[col]);     // (an upper bound: the largest S of the column plus |b|)
        for (int off = 32; off > 0; off >>= 1) sa_max = fmaxf(sa_max, __shfl_xor(sa_max, off, 64));
        if (!(sa_max < INFINITY)) sa_max = INFINITY;
        if (lane == 0) atomicMax(&s_maxabs[kp], __float_as_int(sa_max));   // (non-negative floats order as their bit patterns)
    }
    __syncthreads();

    // ---- selection: wavefront w handles tokens w * 4 .. w * 4 + 3, all four interleaved
    float band;                                                     // twice the error bound of every fp32 logit of this workgroup
    {
        float s_all = 0.f;
#pragma unroll
        for (int p = 0; p < KP; ++p) s_all += __int_as_float(s_maxabs[p]);
        const float err_unit = kErrFactor * (float)(d + 1) * 5.9604645e-8f;   // (d + 1) 2^-24, times the safety factor
        band = 2.f * (err_unit * s_all * 1.0000005f + 1e-30f);
    }
    float cv[kTokW][NC];                                            // the fp32 logits of expert lane + 64 c
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        const int e = lane + 64 * c;
        const float bias = bias_sel[c];
#pragma unroll
        for (int q = 0; q < kTokW; ++q) {
            float l = s_logit[0][wave * kTokW + q][e];
#pragma unroll
            for (int p = 1; p < KP; ++p) l += s_logit[p][wave * kTokW + q][e];
            l += bias;
            if (!(l == l)) l = -INFINITY;                           // a NaN never wins a comparison: rank it last
            cv[q][c] = e < E ? l : -INFINITY;
        }
    }
    float vk[kTokW];                                                // the k-th largest fp32 logit
    {
        unsigned taken[kTokW];
#pragma unroll
        for (int q = 0; q < kTokW; ++q) { taken[q] = 0; vk[q] = -INFINITY; }
        for (int j = 0; j < k; ++j) {
            float bv[kTokW]; int bi[kTokW];
#pragma unroll
            for (int q = 0; q < kTokW; ++q) {
                bv[q] = -INFINITY; bi[q] = kNone;
#pragma unroll
                for (int c = 0; c < NC; ++c) {
                    const int e = lane + 64 * c;
                    if (e < E && !((taken[q] >> c) & 1) && better(cv[q][c], e, bv[q], bi[q])) { bv[q] = cv[q][c]; bi[q] = e; }
                }
            }
            for (int off = 32; off > 0; off >>= 1) {
#pragma unroll
                for (int q = 0; q < kTokW; ++q) {
                    const float ov = __shfl_xor(bv[q], off, 64);
                    const int oi = __shfl_xor(bi[q], off, 64);
                    if (better(ov, oi, bv[q], bi[q])) { bv[q] = ov; bi[q] = oi; }
                }
            }
#pragma unroll
            for (int q = 0; q < kTokW; ++q) {
                if (bi[q] != kNone && (bi[q] & 63) == lane) taken[q] |= 1u << (bi[q] >> 6);   // the owner retires the winner
                vk[q] = bv[q];
            }
        }
    }
    // candidates: fp32 logit >= v_k - band (an expert below that is below the exact k-th largest); their ids in
    // ascending order go to s_cand.  A token is handled here if the bound is finite and the candidates fit.
    int n_cand[kTokW];
    unsigned handled = 0;                                           // bit q: token q's selection is made below
#pragma unroll
    for (int q = 0; q < kTokW; ++q) {
        const int r = wave * kTokW + q;
        const float thr = vk[q] - band;
        int n = 0;
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            const int e = lane + 64 * c;
            const bool in = e < E && cv[q][c] >= thr;
            const unsigned long long m = __ballot(in);
            const int rank = n + __popcll(m & ((1ull << lane) - 1ull));
            if (in && rank < kCand) s_cand[r][rank] = e;
            n += __popcll(m);
        }
        n_cand[q] = n;
        const bool ok = band < INFINITY && n >= k && n <= kCand;
        if (ok) handled |= 1u << q;
        else if (lane == 0 && t0 + r < N) fail[1 + atomicAdd(fail, 1)] = t0 + r;
    }
    __syncthreads();                                                // (s_cand is read by other lanes than its writers)

    // ---- exact logits of the candidates: 16 lanes per token, two candidates per pass
    const int q_mine = lane >> 4, sub = lane & 15;
    int n_mine = 0;
#pragma unroll
    for (int q = 0; q < kTokW; ++q)
        if (q == q_mine) n_mine = ((handled >> q) & 1) ? n_cand[q] : 0;
    int n_most = 0;
#pragma unroll
    for (int q = 0; q < kTokW; ++q) n_most = max(n_most, ((handled >> q) & 1) ? n_cand[q] : 0);
    const int r_mine = wave * kTokW + q_mine;
    const int t_mine = t0 + r_mine;
    const u16* xr = X + (size_t)min(t_mine, N - 1) * d;
    double mine = -INFINITY; int my_e = kNone;                      // lane sub of the token's 16 holds candidate sub
    for (int j = 0; j < n_most; j += 2) {
        const int e0 = j < n_mine ? s_cand[r_mine][j] : -1, e1 = j + 1 < n_mine ? s_cand[r_mine][j + 1] : -1;
        double s0, s1;
        dot2_fp64(xr, WgT + (size_t)max(e0, 0) * d, WgT + (size_t)max(e1, 0) * d, d, sub, s0, s1);
        for (int off = 8; off > 0; off >>= 1) {
            s0 += __shfl_xor(s0, off, 64);
            s1 += __shfl_xor(s1, off, 64);
        }
        if (bg) { s0 += (double)bg[max(e0, 0)]; s1 += (double)bg[max(e1, 0)]; }
        if (!(s0 == s0)) s0 = -INFINITY;
        if (!(s1 == s1)) s1 = -INFINITY;
        if (sub == j && e0 >= 0) { mine = s0; my_e = e0; }
        if (sub == j + 1 && e1 >= 0) { mine = s1; my_e = e1; }
    }
    double lsel[kMaxK]; int isel[kMaxK];
#pragma unroll
    for (int j = 0; j < kMaxK; ++j) {
        if (j >= k) break;
        double bv = mine; int bi = my_e;
        for (int off = 8; off > 0; off >>= 1) {
            const double ov = __shfl_xor(bv, off, 64);
            const int oi = __shfl_xor(bi, off, 64);
            if (better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
        }
        if (bi == my_e) { mine = -INFINITY; my_e = kNone; }         // the owner retires the winner
        lsel[j] = bv; isel[j] = bi;
    }
    double den = 0.0, ex[kMaxK];
#pragma unroll
    for (int j = 0; j < kMaxK; ++j) {
        if (j >= k) break;
        ex[j] = exp(lsel[j] - lsel[0]);
        den += ex[j];
    }
    if (sub == 0 && n_mine > 0 && t_mine < N) {
#pragma unroll
        for (int j = 0; j < kMaxK; ++j) {
            if (j >= k) break;
            topk_idx[(size_t)t_mine * k + j] = isel[j];
            topk_w[(size_t)t_mine * k + j] = (float)(ex[j] / den);
        }
    }
}

// A wavefront per listed token: all E logits in fp64 the same way, a lane keeping those of experts lane, lane + 64, ...;
// then k rounds of a wavefront-wide argmax with ties to the lower expert id.
__global__ __launch_bounds__(256) void gate_fix_kernel(const u16* __restrict__ X, const u16* __restrict__ WgT,
                                                       const float* __restrict__ bg, int d, int E, int k,
                                                       int32_t* __restrict__ topk_idx, float* __restrict__ topk_w,
                                                       const int32_t* __restrict__ fail)
{
    constexpr int kPerLane = kMaxE / 64;    // 16 experts per lane at most
    const int lane = threadIdx.x & 63;
    const int wave_global = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int count = fail[0];
    for (int n = wave_global; n < count; n += kFixWaves) {
        const int t = fail[1 + n];
        const u16* xr = X + (size_t)t * d;
        double l[kPerLane];
#pragma unroll
        for (int c = 0; c < kPerLane; ++c) l[c] = -INFINITY;
        for (int e0 = 0; e0 < E; e0 += 4) {                         // four experts at a time: their loads are in flight together
            double s4[4] = {0.0, 0.0, 0.0, 0.0};
            for (int c = lane; c < d / 8; c += 64) {
                const uint4 xv = *(const uint4*)(xr + c * 8);
                uint4 wv[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) wv[u] = *(const uint4*)(WgT + (size_t)min(e0 + u, E - 1) * d + c * 8);
                const unsigned xs[4] = {xv.x, xv.y, xv.z, xv.w};
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const unsigned ws[4] = {wv[u].x, wv[u].y, wv[u].z, wv[u].w};
#pragma unroll
                    for (int q = 0; q < 4; ++q) {                   // (every expert in the same order: equal gate columns give equal sums)
                        s4[u] = fma((double)__uint_as_float(xs[q] << 16), (double)__uint_as_float(ws[q] << 16), s4[u]);
                        s4[u] = fma((double)__uint_as_float(xs[q] & 0xffff0000u), (double)__uint_as_float(ws[q] & 0xffff0000u), s4[u]);
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int e = e0 + u;
                double v = s4[u];
                for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
                v += (bg && e < E) ? (double)bg[e] : 0.0;
                if (!(v == v)) v = -INFINITY;
#pragma unroll
                for (int c = 0; c < kPerLane; ++c)
                    if (e < E && (e >> 6) == c && (e & 63) == lane) l[c] = v;
            }
        }
        int taken = 0;                                              // bit c: this lane's expert c * 64 + lane is selected
        double lsel[kMaxK]; int isel[kMaxK];
#pragma unroll
        for (int j = 0; j < kMaxK; ++j) {
            if (j >= k) break;
            double bv = -INFINITY; int bi = kNone;
#pragma unroll
            for (int c = 0; c < kPerLane; ++c) {
                const int e = c * 64 + lane;
                if (e < E && !((taken >> c) & 1) && better(l[c], e, bv, bi)) { bv = l[c]; bi = e; }
            }
            for (int off = 32; off > 0; off >>= 1) {
                const double ov = __shfl_xor(bv, off, 64);
                const int oi = __shfl_xor(bi, off, 64);
                if (better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
            }
            if ((bi & 63) == lane && bi < E) taken |= 1 << (bi >> 6);
            lsel[j] = bv; isel[j] = bi;
        }
        double den = 0.0, ex[kMaxK];
#pragma unroll
        for (int j = 0; j < kMaxK; ++j) {
            if (j >= k) break;
            ex[j] = exp(lsel[j] - lsel[0]);
            den += ex[j];
        }
        if (lane == 0) {
#pragma unroll
            for (int j = 0; j < kMaxK; ++j) {
                if (j >= k) break;
                topk_idx[(size_t)t * k + j] = isel[j];
                topk_w[(size_t)t * k + j] = (float)(ex[j] / den);
            }
        }
    }
}

}  // namespace

template <int G>
static void launch_fast(const moe_desc_t& D, const u16* X, const u16* WgT, const float* bg, int32_t* topk_idx, float* topk_w,
                        int32_t* fail, hipStream_t st)
{
    if (!allow_dynamic_lds(gate_bf16_kernel<G>, Lds<G>::kTotal)) return;
    hipLaunchKernelGGL(gate_bf16_kernel<G>, dim3((unsigned)((D.N + kTok - 1) / kTok)), dim3(kWaves * 64), Lds<G>::kTotal, st, X, WgT, bg,
                       D.N, D.d, D.E, D.k, topk_idx, topk_w, fail);
}

// bf16, 17 to 256 experts, and no caller of the stored logits (scores over all experts, balance statistics).
void launch_gate_bf16(const moe_desc_t& D, const void* X, const void* Wg, const float* bg, int32_t* topk_idx, float* topk_w,
                      void* WgT, int32_t* fail, hipStream_t st)
{
    using T = unsigned short;
    const long n = (long)D.d * D.E;
    hipLaunchKernelGGL(gate_prep<T>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, (const T*)Wg, (T*)WgT, D.d, D.E, fail);
    if (D.N == 0) return;
    if (D.E <= 64) launch_fast<64>(D, (const u16*)X, (const u16*)WgT, bg, topk_idx, topk_w, fail, st);
    else if (D.E <= 128) launch_fast<128>(D, (const u16*)X, (const u16*)WgT, bg, topk_idx, topk_w, fail, st);
    else launch_fast<256>(D, (const u16*)X, (const u16*)WgT, bg, topk_idx, topk_w, fail, st);
    hipLaunchKernelGGL(gate_fix_kernel, dim3(kFixWaves / 4), dim3(256), 0, st, (const u16*)X, (const u16*)WgT, bg, D.d, D.E, D.k,
                       topk_idx, topk_w, (const int32_t*)fail);
}

}  // namespace moe
