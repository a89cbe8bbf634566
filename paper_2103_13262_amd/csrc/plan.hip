// Counting, offsets and the stable position of every assignment inside its expert's segment
// (Section 3.2: the samples per expert are counted first and the buffer offsets follow from
// the counts; Section 4: the samples of one expert lie contiguously).  Integer work only.
//
//   plan_hist : per chunk of kPlanChunk assignments, an LDS histogram over experts (small problems: done by
//               plan_scan itself, which saves the launch).
//   plan_scan : one workgroup; column scan over chunks -> counts and per-chunk bases, exclusive
//               scan over experts -> offsets, tile prefix tables for four row-tile heights,
//               experts ordered by descending count.
//   plan_rank : per chunk, each wavefront ranks 64 assignments at a time with ballots (lanes
//               that hold the same expert are found bit by bit), so rows keep assignment order.
#include "common.h"

namespace moe {

__global__ __launch_bounds__(256) void plan_hist(const int32_t* __restrict__ idx, long M, int E,
                                                 int32_t* __restrict__ hist)
{
    __shared__ int sh[kMaxE];
    for (int e = threadIdx.x; e < E; e += 256) sh[e] = 0;
    __syncthreads();
    const long base = (long)blockIdx.x * kPlanChunk;
    for (int q = 0; q < kPlanChunk / 256; ++q) {
        const long a = base + q * 256 + threadIdx.x;
        if (a < M) {
            const int e = idx[a];
            if (e >= 0 && e < E) atomicAdd(&sh[e], 1);
        }
    }
    __syncthreads();
    for (int e = threadIdx.x; e < E; e += 256) hist[(size_t)blockIdx.x * E + e] = sh[e];
}

// Exclusive scans of NV ints per thread over a 1024-thread workgroup, all at once (v[i] -> sum of v[i] over the
// threads below); `total[i]` receives the sums.  Threads n_used and above hold zeros: their wavefronts skip the
// shuffles (the LDS crossbar that carries them is shared by all sixteen).
template <int NV>
__device__ __forceinline__ void block_excl_scan_1024(int (&v)[NV], int (*s_wave)[NV] /*[16][NV]*/, int (&total)[NV], int n_used)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int inc[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) inc[i] = v[i];
    if (wave * 64 < n_used) {
        for (int off = 1; off < 64; off <<= 1) {
#pragma unroll
            for (int i = 0; i < NV; ++i) {
                const int o = __shfl_up(inc[i], off, 64);
                if (lane >= off) inc[i] += o;
            }
        }
    }
    if (lane == 63) {
#pragma unroll
        for (int i = 0; i < NV; ++i) s_wave[wave][i] = inc[i];
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        int wbase = 0, tot = 0;
        for (int w = 0; w * 64 < n_used; ++w) {
            const int c = s_wave[w][i];
            if (w < wave) wbase += c;
            tot += c;
        }
        total[i] = tot;
        v[i] = wbase + inc[i] - v[i];
    }
}

constexpr int kFusedHistInts = 8192;   // chunk histograms that plan_scan builds itself when they fit (32 KB of LDS)

// idx == nullptr: the chunk histograms were written to `hist` by plan_hist.  Otherwise (nb * E <= kFusedHistInts)
// this workgroup counts the assignments itself, into LDS, and saves that launch.
__global__ __launch_bounds__(1024) void plan_scan(const int32_t* __restrict__ idx, int32_t* __restrict__ hist, int nb,
                                                  int E, long M, int32_t* __restrict__ counts,
                                                  int32_t* __restrict__ offsets, int32_t* __restrict__ tileP,
                                                  int32_t* __restrict__ order, int32_t* __restrict__ cls,
                                                  int32_t* __restrict__ zeros)
{
    // the control block: the page read in place of masked rows and the control words of the grouped products
    if (threadIdx.x < kCtlWords) zeros[threadIdx.x] = 0;
    __shared__ __align__(16) int s_cnt[kMaxE];
    __shared__ int s_wave[16][3 + kNumTileHeights];
    __shared__ int s_hist[kFusedHistInts];
    const int e = threadIdx.x;
    int cnt = 0;
    if (idx) {
        for (int i = threadIdx.x; i < nb * E; i += 1024) s_hist[i] = 0;
        __syncthreads();
        for (long a0 = 0; a0 < M; a0 += 8 * 1024) {       // eight loads in flight per thread
            int ev[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const long a = a0 + u * 1024 + threadIdx.x;
                ev[u] = a < M ? idx[a] : -1;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const long a = a0 + u * 1024 + threadIdx.x;
                if (ev[u] >= 0 && ev[u] < E) atomicAdd(&s_hist[(int)(a / kPlanChunk) * E + ev[u]], 1);
            }
        }
        __syncthreads();
        if (e < E) {
            for (int b = 0; b < nb; ++b) {                // exclusive bases inside the expert, for plan_rank
                const int v = s_hist[b * E + e];
                hist[(size_t)b * E + e] = cnt;
                cnt += v;
            }
            counts[e] = cnt;
        }
    } else if (e < E) {
        // chunk histograms -> exclusive bases inside the expert, eight chunks at a time so that their loads are in
        // flight together (one after the other, each load would wait for the store before it)
        for (int b0 = 0; b0 < nb; b0 += 8) {
            int v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = hist[(size_t)min(b0 + u, nb - 1) * E + e];
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (b0 + u < nb) {
                    hist[(size_t)(b0 + u) * E + e] = cnt;
                    cnt += v[u];
                }
        }
        counts[e] = cnt;
    }
    s_cnt[e] = e < E ? cnt : -1;
    // one pass of scans: offsets, the tile prefix tables of every tile height, the two size classes of every expert's rows
    int nbig = cnt / kClsBigRows, last = cnt - nbig * kClsBigRows;
    if (last > kClsSmallRows) { ++nbig; last = 0; }
    constexpr int NV = 3 + kNumTileHeights;
    int sc[NV], total[NV];
    sc[0] = cnt;
    sc[1] = e < E ? nbig : 0;
    sc[2] = e < E && last > 0 ? 1 : 0;
#pragma unroll
    for (int q = 0; q < kNumTileHeights; ++q) sc[3 + q] = e < E ? (cnt + tile_height(q) - 1) / tile_height(q) : 0;
    block_excl_scan_1024<NV>(sc, s_wave, total, E);
    const int off = sc[0];
    if (e < E) {
        offsets[e] = off;
        cls[kClsCountsBig * (E + 1) + e] = min(cnt, nbig * kClsBigRows);
        cls[kClsCountsSmall * (E + 1) + e] = last;
        cls[kClsOffsetsSmall * (E + 1) + e] = off + nbig * kClsBigRows;
        cls[kClsPBig * (E + 1) + e] = sc[1];
        cls[kClsPSmall * (E + 1) + e] = sc[2];
#pragma unroll
        for (int q = 0; q < kNumTileHeights; ++q) tileP[q * (E + 1) + e] = sc[3 + q];
    }
    if (e == 0) {
        offsets[E] = total[0];
        cls[kClsPBig * (E + 1) + E] = total[1];
        cls[kClsPSmall * (E + 1) + E] = total[2];
#pragma unroll
        for (int q = 0; q < kNumTileHeights; ++q) tileP[q * (E + 1) + E] = total[3 + q];
    }
    __syncthreads();
    int rank = 0;                         // experts by descending count, ties by ascending id
    if (e < E) {
#pragma unroll 4
        for (int o = 0; o < E; o += 4) {          // (the counts past E are -1: they never rank before an expert)
            const int4 c = *(const int4*)&s_cnt[o];
            rank += (c.x > cnt || (c.x == cnt && o < e)) ? 1 : 0;
            rank += (c.y > cnt || (c.y == cnt && o + 1 < e)) ? 1 : 0;
            rank += (c.z > cnt || (c.z == cnt && o + 2 < e)) ? 1 : 0;
            rank += (c.w > cnt || (c.w == cnt && o + 3 < e)) ? 1 : 0;
        }
        order[rank] = e;
    }
    // Can the weight-gradient products give every XCD whole experts (expert of rank r to XCD r%8, every other
    // group of eight reversed)?  Then each operand panel is fetched by one XCD only.  Only if the reduction blocks
    // that each XCD would get stay within 10 % of the mean; the answer is control word kCtlByExpert.
    __shared__ int s_xcd[8], s_big;
    if (threadIdx.x < 8) s_xcd[threadIdx.x] = 0;
    if (e < E && rank == 0) s_big = cnt;      // the largest expert
    __syncthreads();
    if (e < E) atomicAdd(&s_xcd[(rank >> 3) & 1 ? 7 - (rank & 7) : rank & 7], (cnt + 63) / 64);
    __syncthreads();
    if (threadIdx.x == 0) {
        int mx = 0, sum = 0;
        for (int x = 0; x < 8; ++x) { mx = max(mx, s_xcd[x]); sum += s_xcd[x]; }
        zeros[kCtlByExpert] = (E >= 8 && (long)mx * 80 <= (long)sum * 11) ? 1 : 0;
        // Strongly skewed sizes (largest expert above three times the mean): the weight-gradient products hand out
        // their tiles on demand instead of in fixed rounds; (control word kCtlSkewed).
        zeros[kCtlSkewed] = (E >= 2 && (long)s_big * E > 3 * M) ? 1 : 0;
    }
}

__global__ __launch_bounds__(256) void plan_rank(const int32_t* __restrict__ idx, long M, int E, int nbits,
                                                 const int32_t* __restrict__ base, const int32_t* __restrict__ offsets,
                                                 int32_t* __restrict__ pos, int32_t* __restrict__ perm)
{
    __shared__ int wcnt[4][kMaxE];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int e = threadIdx.x; e < E; e += 256)
        for (int w = 0; w < 4; ++w) wcnt[w][e] = 0;
    __syncthreads();
    const long cbase = (long)blockIdx.x * kPlanChunk + wave * 256;
    int ev[4];
    for (int s = 0; s < 4; ++s) {
        const long a = cbase + s * 64 + lane;
        int e = -1;
        if (a < M) {
            e = idx[a];
            if (e < 0 || e >= E) e = -1;  // cannot happen for indices written by the gate kernel
        }
        ev[s] = e;
        if (e >= 0) atomicAdd(&wcnt[wave][e], 1);
    }
    __syncthreads();
    for (int e = threadIdx.x; e < E; e += 256) {
        int run = base[(size_t)blockIdx.x * E + e] + offsets[e];
        for (int w = 0; w < 4; ++w) {
            const int c = wcnt[w][e];
            wcnt[w][e] = run;
            run += c;
        }
    }
    __syncthreads();
    for (int s = 0; s < 4; ++s) {
        const int e = ev[s];
        const bool valid = e >= 0;
        unsigned long long mask = __ballot(valid);
        for (int b = 0; b < nbits; ++b) {
            const bool bit = valid && ((e >> b) & 1);
            const unsigned long long bal = __ballot(bit);
            mask &= bit ? bal : ~bal;
        }
        int p = 0;
        if (valid) {
            const int rank = __popcll(mask & ((1ull << lane) - 1ull));
            p = wcnt[wave][e] + rank;
            const long a = cbase + s * 64 + lane;
            pos[a] = p;
            perm[p] = (int32_t)a;
        }
        __syncthreads();  // every lane has read its counter before the group leader advances it
        if (valid && (mask >> lane) == 1ull) wcnt[wave][e] = p + 1;
        __syncthreads();
    }
}

void launch_plan(const moe_desc_t& D, const WsLayout& L, const int32_t* topk_idx, int32_t* counts,
                 int32_t* offsets, int32_t* pos, int32_t* perm, char* ws, hipStream_t st)
{
    const long M = (long)D.N * D.k;
    int32_t* hist = (int32_t*)(ws + L.hist);
    int32_t* tileP = (int32_t*)(ws + L.tileP);
    int32_t* order = (int32_t*)(ws + L.order);
    int nbits = 0;
    while ((1 << nbits) < D.E) ++nbits;
    const bool fused = L.nb > 0 && (long)L.nb * D.E <= kFusedHistInts;
    if (L.nb > 0 && !fused) hipLaunchKernelGGL(plan_hist, dim3(L.nb), dim3(256), 0, st, topk_idx, M, D.E, hist);
    hipLaunchKernelGGL(plan_scan, dim3(1), dim3(1024), 0, st, fused ? topk_idx : (const int32_t*)nullptr, hist, L.nb, D.E,
                       M, counts, offsets, tileP, order, (int32_t*)(ws + L.cls), (int32_t*)(ws + L.zeros));
    if (L.nb > 0)
        hipLaunchKernelGGL(plan_rank, dim3(L.nb), dim3(256), 0, st, topk_idx, M, D.E, nbits, (const int32_t*)hist,
                           (const int32_t*)offsets, pos, perm);
}

}  // namespace moe
