// Grouped bf16 matrix products on the matrix cores, persistent form.
//
// One workgroup per compute unit stays resident for the whole launch and walks a list of work items.
// A work item is an output tile (BM x BN) together with a range of its reduction blocks (BK deep):
//   * whole tiles, handed out in rounds (workgroup j of an XCD takes tile j, j + W, ... of the XCD's share), and
//   * for the tiles left over after the last full round, equal pieces of their reduction ("stream-K"): the
//     left-over tiles of an XCD are laid end to end, block by block, and cut into one contiguous range per
//     workgroup.  A range that ends inside a tile yields a partial sum, written in fp32 to a per-workgroup
//     buffer; a range that begins inside a tile first adds the partial sum of the workgroup before it (which
//     holds the preceding blocks of that tile), so the sum runs along the tile's workgroups in ascending
//     order (a fixed order: results do not depend on timing) and the workgroup whose range holds the tile's
//     last block writes the tile.  Every workgroup handles the piece at the end of its range first, and a
//     workgroup waits only for the one numbered just below it, so the waits cannot form a cycle.
// The rows kinds compute an expert's whole blocks of 256 rows in 256 x 256 tiles and its last piece (at most 128 rows)
// in 128 x 512 tiles, from the plan step's size-class tables (ggemm_cls_kernel); many small experts: 64 x 256 tiles.
// The weight gradients (whole tiles only: their reduction runs over an expert's rows) take their tiles in fixed
// rounds too, or - when the experts' sizes are strongly skewed, or when they follow another product inside one
// launch (ggemm_pair_kernel) - from counters in memory, on demand.
// Operands travel from global memory straight into an LDS ring (global_load_lds_dwordx4), the first blocks
// of the next work item are requested before the epilogue of the current one, and the epilogue runs through
// a small LDS patch of its own so that it does not disturb the ring.
//
// Workgroup: WM x WN wavefronts, each owning TM x TN accumulators of v_mfma_f32_32x32x16_bf16.
//
// LDS layouts of the ring (each wave-level load fills one contiguous 1 KB piece, lane p -> byte 16*p, so a
// layout is chosen by choosing which global 16-byte chunk each lane fetches):
//   k-contiguous source ([row][k]):  LDS row = 2*BK bytes; 16-byte chunk c of row r sits at position
//       c ^ swz(r); operand reads are ds_read_b128 and free of bank conflicts.
//   row-contiguous source ([k][row], the reduction index is the slow one: weights in the forward products,
//       both operands of the weight gradients): an LDS row is one k-row (512 bytes: every k-row starts at
//       bank 0), chunk c of k-row k sits at position swap13(c) ^ 2*(k&3), where swap13 exchanges bits 1 and 3 of
//       the chunk number; operands are gathered with ds_read_b64_tr_b16.  One such read takes, per 16 lanes,
//       2 chunks of each of 4 k-rows, and the next 16 lanes take the 2 chunks beside them: the positions of 16
//       lanes are distinct modulo 8 and those of 32 lanes distinct modulo 16, so the read is free of bank
//       conflicts whether the LDS serves 128 or 256 bytes per clock.
// Rows / columns outside a tile's valid extent are fetched from a clamped (valid) address and their results
// are never stored.  (Not requesting them at all changes nothing measurable: a block of a tile with few valid
// rows takes as long as the requests for the other operand take to arrive.)  Reduction indices past the end are
// fetched from a page of zeros.
//
// The Gaussian factors of GeLU and GeLU' are looked up at the bf16 value zb that is stored as the
// pre-activation, so they are functions of 16 bits: an LDS table indexed by the bit pattern (built from erfc /
// exp at launch) gives Phi(zb) resp. Phi(zb) + zb phi(zb) exactly for 2^-11 <= |zb| < 8 and the nearest table
// entry outside (|error| < 4e-4).  Forward: H = z (Phi(zb) + (z - zb) phi(zb)) with z the fp32 accumulator: the
// table's value at the rounded argument, carried back to z along the slope.  (Without the slope term H is off by up
// to z^2 phi(z) 2^-9 < 6e-4, a fraction of H's own bf16 rounding, but enough to raise the error of the gate's
// gradient by half in shapes with few tokens per expert.)
#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <mutex>
#include <type_traits>
#include <utility>
#include <vector>

#include "common.h"

namespace moe {
namespace sk {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef unsigned short u16;
#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))

constexpr int kMinSplitDepth = 16 * 64;         // a stream-K piece is at least this deep (16 blocks of 64): handing a partial sum on costs
                                                // about as much time as 6 such blocks, and the hand-overs of one tile form a chain
constexpr int kActLo = (127 - 11) << 7;         // bf16 bit pattern of 2^-11
constexpr int kActHi = (127 + 3) << 7;          // bf16 bit pattern of 2^3
constexpr int kActEntries = kActHi - kActLo;    // table entries per sign
constexpr int kSpinLimit = 1 << 20;             // bounded wait for a partial sum (on the order of a second)

// Results can leave the chip as streaming (non-temporal) stores: none of them is read again by the launch that writes
// it, and written the ordinary way they displace operand panels from the caches.  Measured on one machine, A against
// B: -2 % per step on the paper's shape (134 MB of weights per product), -6 % with 64 or 256 experts, the weight
// gradients' stores mattering most; but +1.5 to +3 % with 1, 2 or 4 experts of that width (8 to 32 MB), whose weights
// stay in the 32 MB of L2 whatever the stores do, so that what counts is how fast the stores are taken.  The host
// decides per launch (GemmArgs::stream_out): streaming when one product's weights exceed 48 MB.
typedef __attribute__((ext_vector_type(4))) unsigned u32x4_t;
__device__ __forceinline__ void store_out(uint4* p, const uint4 v, bool streaming)
{
    if (streaming) {
        const u32x4_t w = {v.x, v.y, v.z, v.w};
        __builtin_nontemporal_store(w, (u32x4_t*)p);
    } else *p = v;
}
__device__ __forceinline__ int swap13(int c) { return (c & ~10) | ((c & 2) << 2) | ((c & 8) >> 2); }

template <int BK> __device__ __forceinline__ int swz(int r)
{
    if constexpr (BK == 32) return ((r >> 1) & 3) ^ ((r >> 3) & 1);
    else if constexpr (BK == 64) return (r >> 1) & 7;
    else return r & 15;   // 256-byte rows: every row starts at bank 0, 16 rows take 16 different chunk positions
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
    static constexpr int RING = STAGES * STAGE_BYTES;
    static constexpr int TNG = TN < 2 ? TN : 2;               // accumulator columns that pass through the patch together
    static constexpr int PITCH = TNG * 32 + 8;                // floats per patch row: rows 4 apart are 32 banks apart
    static constexpr int PATCH_BYTES = NW * 8 * PITCH * 4;    // 8 rows per wave
    static constexpr bool TABLE = KIND == kRowsNN_GeLU || KIND == kRowsNT_dGeLU;
    static constexpr int TABLE_BYTES = TABLE ? 2 * kActEntries * 4 : 0;
    static constexpr int NEXT_BYTES = KIND == kColsT ? 16 : 0;   // the tile index handed out on demand
    static constexpr int SMEM = RING + PATCH_BYTES + TABLE_BYTES + NEXT_BYTES;
    static_assert(A_BYTES % (1024 * NW) == 0 && B_BYTES % (1024 * NW) == 0, "tile must split evenly over waves");
    static_assert(SMEM <= 160 * 1024, "LDS budget");
};

// Entry i of the activation table: Phi(z) (forward) or Phi(z) + z phi(z) (backward) at the bf16 value whose
// magnitude pattern is kActLo + i % kActEntries and whose sign is i / kActEntries.
template <int KIND> __device__ __forceinline__ float act_entry(int i)
{
    const int s = i >= kActEntries ? 1 : 0;
    const float z = bf16_to_f32((u16)((i - s * kActEntries + kActLo) | (s << 15)));
    const float cdf = 0.5f * erfcf(-z * 0.70710678118654752f);
    if constexpr (KIND == kRowsNN_GeLU) return cdf;
    else return cdf + z * expf(-0.5f * z * z) * 0.39894228040143268f;
}
__device__ __forceinline__ int act_index(unsigned zb)   // zb: bf16 bit pattern in the low 16 bits
{
    int t = (int)(zb & 0x7fffu);
    t = min(max(t, kActLo), kActHi - 1);
    return t - kActLo + (int)((zb >> 15) & 1u) * kActEntries;
}

// Per-lane source pointers of one operand for reduction block 0 (advanced by the caller) and the
// reduction offset inside a block that the lane's chunk starts at (krow).
//   !TRANS: src[row][k]; one load covers 64 / (BK/8) rows.
//    TRANS: src[k][row]; CPR = R/8 chunks per k-row; lane p of load j covers k-row j*(64/CPR) + p/CPR.
//   gather (!TRANS only): row r of the tile is the source's row gather[row0 + r] / div instead of row r.
template <bool TRANS, int R, int NW, int L, int BK>
__device__ __forceinline__ void setup_ptrs(const u16* base, long ld, int valid, int wave, int lane, const u16* (&ptr)[L],
                                           int (&krow)[L], const int32_t* gather = nullptr, long row0 = 0, int div = 1)
{
#pragma unroll
    for (int i = 0; i < L; ++i) {
        const int j = wave + i * NW;
        if constexpr (!TRANS) {
            constexpr int CK = BK / 8;
            int row = j * (64 / CK) + lane / CK;
            const int c = (lane % CK) ^ swz<BK>(row);
            row = row < valid ? row : valid - 1;
            const long src_row = gather ? (long)(gather[row0 + row] / div) : (long)row;
            ptr[i] = base + src_row * ld + c * 8;
            krow[i] = c * 8;
        } else {
            constexpr int CPR = R / 8;
            static_assert(CPR >= 16 && 64 % CPR == 0, "the position code needs 16 chunks per k-row");
            const int kr = j * (64 / CPR) + lane / CPR;
            int c = swap13((lane % CPR) ^ (2 * (kr & 3)));
            c = c * 8 < valid ? c : 0;
            ptr[i] = base + (long)kr * ld + c * 8;
            krow[i] = kr;
        }
    }
}

// One work item (all fields are uniform over the workgroup).
struct Item {
    const u16* A; long lda;
    const u16* B; long ldb;
    size_t c_off;
    int Mt, Nt, Kt;       // valid rows / columns of the tile, reduction length
    int kb0, kb1;         // reduction blocks [kb0, kb1) of the tile
    int owner;            // the range holds the tile's last block: this workgroup writes the tile
    size_t b_off;         // rows kinds: expert * Nout + first column (where the tile's bias values start)
    long row0;            // rows kinds: first row of the tile in the expert-contiguous order
};

struct Fin {              // what finishing an item needs once the streams have moved on to the next one
    size_t c_off, b_off;
    int Mt, Nt, owner;
    long row0;
};

// CLS: 0 = all rows of every expert (tables counts / offsets / tileP); 1 = the rows in whole blocks of
// kClsBigRows, 2 = the experts' last pieces (the plan step's size-class tables; rows kinds only).
// Of every XCD's workgroups, those numbered wj_base .. wj_base + wj_count - 1 take part (wj_count <= 0: all); the
// others return at once.
template <int KIND, int WM, int WN, int TM, int TN, int STAGES, int BK, int CLS = 0>
__device__ __forceinline__ void ggemm_sk_body(const GemmArgs& g, int ntm, int ntn, int wj_base = 0, int wj_count = 0)
{
    using C = Cfg<KIND, WM, WN, TM, TN, STAGES, BK>;
    static_assert(CLS == 0 || (KIND != kColsT && C::BM == (CLS == 1 ? kClsBigRows : kClsSmallRows)), "size class and tile height");
    const int32_t* const counts_ = CLS == 0 ? g.counts : g.cls + (CLS == 1 ? kClsCountsBig : kClsCountsSmall) * (g.E + 1);
    const int32_t* const offsets_ = CLS == 2 ? g.cls + kClsOffsetsSmall * (g.E + 1) : g.offsets;
    constexpr int BM = C::BM, BN = C::BN, NT = C::NT, PITCH = C::PITCH;
    extern __shared__ __align__(1024) char smem[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;

    // split tiles of the last pieces' class use the second set of partial-sum buffers and flags: a workgroup that
    // has moved on to that class must not overwrite what its successor has yet to read of the first
    constexpr int kPhase = CLS == 2 ? 1 : 0;
    const int sk_slot = kPhase * kMaxPersistentWgs + (int)blockIdx.x;
    float* patch = (float*)(smem + C::RING) + wave * (8 * PITCH);
    const float* act = (const float*)(smem + C::RING + C::PATCH_BYTES);

    const long long probe_cycles0 = clock64(), probe_ticks0 = wall_clock64();

    // ---------------- schedule of this workgroup ----------------
    const int xcd = blockIdx.x & 7, wj = (int)(blockIdx.x >> 3) - wj_base, W = wj_count > 0 ? wj_count : (int)(gridDim.x >> 3);
    if (wj < 0 || wj >= W) return;
    const int32_t* P = CLS == 0 ? g.tileP + tile_height_index(BM) * (g.E + 1)
                                : g.cls + (CLS == 1 ? kClsPBig : kClsPSmall) * (g.E + 1);
    long start = 0, n_dp = 0;        // rows kinds: first tile of this XCD's share; number of whole-tile items
    int rem = 0, Wp = 0;             // left-over tiles of this XCD; workgroups taking part in their reduction split
    int row_f = 1;                   // left-over tiles cut into this many row slices instead
    bool row_item = false;           // this workgroup still has to do row slice wj % row_f of left-over tile wj / row_f
    int nkT = 0;                     // rows kinds: reduction blocks per tile
    int sk_a = 0, sk_cur = 0;        // stream-K blocks of this workgroup not yet done: [sk_a, sk_cur)
    long dp_i, dp_stride;            // next whole-tile item and the stride to the one after
    int tpe = 0, per = 0;            // weight gradients: tiles per expert, and per expert and XCD
    bool by_expert = false;          // weight gradients: every XCD works on whole experts (decided by the plan step)
    bool dynamic = false;            // weight gradients: tiles are taken from a per-XCD counter instead of in rounds
    long n_static = 0;               // ... from this item of the list on; the items before it go in fixed rounds
    int32_t* dyn_ctr = nullptr;      // this workgroup's counter (one per XCD, or one for all when tiles are not split by XCD)
    int& s_next = *(int*)(smem + C::RING + C::PATCH_BYTES + C::TABLE_BYTES);   // (weight gradients only)
    if constexpr (KIND != kColsT) {
        const long T = (long)P[g.E] * ntn;
        const long base = T >> 3;
        const int extra = (int)(T & 7);
        const long n_x = base + (xcd < extra ? 1 : 0);
        start = xcd * base + min(xcd, extra);
        nkT = (g.K + BK - 1) / BK;
        rem = (int)(n_x % W);
        if (rem * 10 >= W * 9) rem = 0;       // a nearly full last round is not worth splitting
        n_dp = n_x - rem;
        dp_i = wj; dp_stride = W;
    } else {
        tpe = ntm * ntn;
        by_expert = *g.by_expert != 0;
        if (by_expert) { n_dp = (long)((g.E + 7) / 8) * tpe; dp_i = wj; dp_stride = W; }
        else if ((tpe & 7) == 0) { per = tpe >> 3; n_dp = (long)g.E * per; dp_i = wj; dp_stride = W; }
        else { n_dp = (long)g.E * tpe; dp_i = blockIdx.x; dp_stride = gridDim.x; }
        // A round of tiles can span several experts; when their sizes are strongly skewed, fixed rounds leave the
        // workgroups that got the largest experts' tiles far behind.  Then the list (longest reductions first)
        // is handed out on demand from a counter.
        // (with a whole round inside one expert the fixed rounds are balanced already)
        // A launch that follows another product inside one kernel (on_demand) always does: its workgroups
        // arrive at different times.
        const bool skewed = *g.skewed != 0;
        dynamic = g.on_demand || (!by_expert && (per == 0 || per < W) && skewed);
        dyn_ctr = g.dyn_counters + (by_expert || per ? xcd : 0);
        // An index from the counter costs a round trip to memory (about 2 us).  Sizes that are not skewed need the
        // counter only to even out the workgroups' different arrival times: all but the last two rounds stay fixed.
        if (dynamic && !skewed) n_static = max(0L, n_dp / dp_stride - 2) * dp_stride;
    }

    // Tile number L (rows kinds) -> expert, row block inside the expert, column block.  Order inside an expert:
    // groups of up to GM row blocks; inside a group the row block runs fastest, then the column block, so that
    // tiles that run at the same time on one XCD share operand panels.
    auto locate = [&](long L, int& e, int& mt, int& nt) {
        int lo = 0, hi = g.E;
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if ((long)P[mid] * ntn <= L) lo = mid; else hi = mid;
        }
        e = lo;
        const int mte = P[e + 1] - P[e];
        const int local = (int)(L - (long)P[e] * ntn);
        constexpr int GM = 8;
        const int full = mte / GM, per_group = GM * ntn;
        const int gi = local / per_group;
        if (gi < full) {
            const int r = local - gi * per_group;
            nt = r / GM;
            mt = gi * GM + (r - nt * GM);
        } else {
            const int remm = mte - full * GM;
            const int r = local - full * per_group;
            nt = r / remm;
            mt = full * GM + (r - nt * remm);
        }
    };
    // slice s of f: only rows s*BM/f .. (s+1)*BM/f - 1 of the tile (f = 1: the whole tile)
    auto decode_rows = [&](long L, Item& it, int slice = 0, int f = 1) {
        int e, mt, nt;
        locate(L, e, mt, nt);
        const int rows_per = BM / f, row_off = slice * rows_per;
        const long r0 = (long)offsets_[e] + (long)mt * BM + row_off;
        const int n0 = nt * BN;
        it.A = (const u16*)g.A + (g.a_gather ? 0 : r0 * g.K);  it.lda = g.K;   // (gathered rows: the base, see setup_ptrs)
        it.row0 = r0;
        const u16* Be = (const u16*)g.B + (size_t)e * g.K * g.Nout;
        if constexpr (C::B_TRANS) { it.B = Be + n0; it.ldb = g.Nout; }
        else                      { it.B = Be + (size_t)n0 * g.K; it.ldb = g.K; }
        it.c_off = (size_t)r0 * g.Nout + n0;
        it.b_off = (size_t)e * g.Nout + n0;
        it.Mt = min(rows_per, counts_[e] - mt * BM - row_off);  it.Nt = min(BN, g.Nout - n0);  it.Kt = g.K;
    };
    if constexpr (KIND != kColsT) {
        if (rem && g.whole_tiles) {
            // another product follows in this launch and takes up the workgroups that have nothing left to do here:
            // the left-over tiles are computed whole, one per workgroup (no partial sums, no slices)
            row_f = 1;
            row_item = wj < rem;
        } else if (rem) {
            constexpr int kMinSplitBlocks = kMinSplitDepth / BK;
            if (nkT >= 2 * kMinSplitBlocks) {
                // long reductions: the left-over tiles' blocks, laid end to end, in equal contiguous ranges.  (Ranges
                // of equal estimated time instead - blocks of tiles with few valid rows are cheaper - change nothing
                // measurable: such a block still costs 7/8 of a full one, the operand loads set the pace.)
                const int S = rem * nkT;
                Wp = min(W, max(1, S / kMinSplitBlocks));
                if (wj < Wp) { sk_a = (int)((long)wj * S / Wp); sk_cur = (int)((long)(wj + 1) * S / Wp); }
            } else {
                // short reductions: a hand-over of partial sums would cost as much as the piece itself; when at most
                // half of the workgroups would get a left-over tile, the tiles are cut by rows instead (no partial sums)
                row_f = rem * 4 <= W && BM >= 128 ? 4 : rem * 2 <= W && BM >= 64 ? 2 : 1;
                row_item = wj < rem * row_f;
            }
        }
    }
    auto next_item = [&](Item& it) -> bool {
        if constexpr (KIND != kColsT) {
            if (row_item) {
                row_item = false;
                decode_rows(start + wj / row_f, it, wj % row_f, row_f);
                it.kb0 = 0;  it.kb1 = nkT;  it.owner = 1;
                if (it.Mt > 0) return true;      // (a slice past the tile's last row holds nothing)
            }
            if (sk_cur > sk_a) {       // stream-K pieces, last one first
                const int tt = (sk_cur - 1) / nkT;
                const int seg0 = max(sk_a, tt * nkT);
                it.kb0 = seg0 - tt * nkT;  it.kb1 = sk_cur - tt * nkT;
                it.owner = it.kb1 == nkT;
                sk_cur = seg0;
                decode_rows(start + tt, it);
                return true;
            }
            if (dp_i < n_dp) {
                decode_rows(start + rem + dp_i, it);
                dp_i += dp_stride;
                it.kb0 = 0;  it.kb1 = nkT;  it.owner = 1;
                return true;
            }
            return false;
        } else {
            // Tiles are listed by descending reduction length (experts by descending row count).  Rounds alternate
            // direction, so the workgroup that got the longest tile of one round gets the shortest of the next.
            // Which tiles an XCD gets: when the experts' sizes allow it (by_expert), whole experts - the expert of
            // rank r goes to XCD r%8, every other group of eight reversed - so that each operand panel is fetched
            // into one L2 only; otherwise an eighth of every expert's tiles.
            int ord, q;
            if (dynamic) {
                // (agent-scope atomic: correct wherever the workgroups run; which tile a workgroup computes does not
                // change the tile's value, so results stay bit-for-bit repeatable)
                // (asking for the index one tile ahead, to hide the atomic's round trip, measured slower)
                for (;;) {
                    long item;
                    if (dp_i < n_static) {        // fixed rounds, alternating direction
                        const long round = dp_i / dp_stride, lanepos = dp_i - round * dp_stride;
                        item = round * dp_stride + ((round & 1) ? dp_stride - 1 - lanepos : lanepos);
                        dp_i += dp_stride;
                    } else {
                        if (tid == 0) s_next = __hip_atomic_fetch_add(dyn_ctr, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        __syncthreads();
                        item = n_static + s_next;
                        __syncthreads();          // every wave has read it before the next fetch overwrites it
                    }
                    if (item >= n_dp) return false;
                    if (by_expert) {
                        const int grp = (int)(item / tpe);
                        ord = 8 * grp + ((grp & 1) ? 7 - xcd : xcd);
                        q = (int)(item - (long)grp * tpe);
                        if (ord >= g.E) continue; // (the last group of eight may be incomplete)
                    } else if (per) { ord = (int)(item / per); q = xcd * per + (int)(item - (long)ord * per); }
                    else            { ord = (int)(item / tpe); q = (int)(item - (long)ord * tpe); }
                    break;
                }
            } else
            for (;;) {
                const long round = dp_i / dp_stride, lanepos = dp_i - round * dp_stride;
                const long item = round * dp_stride + ((round & 1) ? dp_stride - 1 - lanepos : lanepos);
                if (round * dp_stride >= n_dp) return false;
                dp_i += dp_stride;
                if (item >= n_dp) return false;   // (only in the last round)
                if (by_expert) {
                    const int grp = (int)(item / tpe);
                    ord = 8 * grp + ((grp & 1) ? 7 - xcd : xcd);
                    q = (int)(item - (long)grp * tpe);
                    if (ord >= g.E) continue;     // (the last group of eight may be incomplete)
                } else if (per) { ord = (int)(item / per); q = xcd * per + (int)(item - (long)ord * per); }
                else            { ord = (int)(item / tpe); q = (int)(item - (long)ord * tpe); }
                break;
            }
            const int e = g.order[ord];
            const int m0 = (q / ntn) * BM, n0 = (q % ntn) * BN;
            const long off = g.offsets[e];
            it.A = (const u16*)g.A + off * g.K + m0;     it.lda = g.K;
            it.B = (const u16*)g.B + off * g.Nout + n0;  it.ldb = g.Nout;
            it.c_off = ((size_t)e * g.K + m0) * g.Nout + n0;
            it.b_off = 0;
            it.Mt = min(BM, g.K - m0);  it.Nt = min(BN, g.Nout - n0);  it.Kt = g.counts[e];
            it.kb0 = 0;  it.kb1 = (it.Kt + BK - 1) / BK;  it.owner = 1;
            return true;
        }
    };

    // ---------------- global -> LDS streams ----------------
    const u16* pa[C::LA]; int ka[C::LA];
    const u16* pb[C::LB]; int kb[C::LB];
    long stepA = 0, stepB = 0;
    int Kt = 0, kb0 = 0;                     // of the item whose loads are being issued
    const u16* zeros = (const u16*)g.zeros + lane * 8;
    // reduction indices past Kt are read from the zero page: always possible for the weight gradients (Kt = rows
    // of the expert), and for the other kinds only when a block is deeper than the 32 that divides every width
    constexpr bool KMASK = KIND == kColsT || BK > 32;
    // Weight panels that one tile only will read (an expert's last piece; experts of at most 64 rows) are requested as
    // streaming data, so that they do not push the panels other tiles share out of the caches.  Which products gain is
    // measured, not derived (same-machine A/B runs): with many small experts the backward products (-9 % and -11 % per
    // launch, the forward ones lose 7-10 %); for the last pieces all but dZ (C2: FC1, FC2 -4 %, dZ + 7 %).  Marking every
    // operand load that way costs 11-25 % per step: the re-use of operands out of L2 is what the main loop lives on.
    constexpr bool kStreamB = ((KIND == kRowsNT || KIND == kRowsNT_dGeLU) && BM == 64) ||
                              (KIND != kColsT && KIND != kRowsNT_dGeLU && CLS == 2);
    // The loads are written as inline assembly so that the compiler does not serialise them against the LDS
    // reads of other ring slots; the ordering is enforced by the explicit vmcnt waits and barriers below.
    const unsigned lds_base = (unsigned)(uintptr_t)LDS_PTR(char, smem);
    // One wave-level load (index l of the LA + LB loads this wave owns per block) of the item's block number
    // li (counted from kb0) into ring slot li % STAGES.  l is a compile-time constant at every call site.
    auto issue_one = [&](int li, auto lc) {
        constexpr int l = decltype(lc)::value;
        const unsigned sA = lds_base + (li % STAGES) * C::STAGE_BYTES + wave * 1024;
        if constexpr (l < C::LA) {
            const u16* src = pa[l];
            if constexpr (KMASK) src = ((kb0 + li) * BK + ka[l] < Kt) ? src : zeros;
            asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off"
                         :: "s"(sA + l * C::NW * 1024), "v"(src) : "memory");
            pa[l] += stepA;
        } else {
            constexpr int i = l - C::LA;
            const u16* src = pb[i];
            if constexpr (KMASK) src = ((kb0 + li) * BK + kb[i] < Kt) ? src : zeros;
            if constexpr (kStreamB)
                asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off nt"
                             :: "s"(sA + C::A_BYTES + i * C::NW * 1024), "v"(src) : "memory");
            else
                asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off"
                             :: "s"(sA + C::A_BYTES + i * C::NW * 1024), "v"(src) : "memory");
            pb[i] += stepB;
        }
    };
    auto issue = [&](int li) {   // all loads of one block at once
        [&]<int... L>(std::integer_sequence<int, L...>) {
            (issue_one(li, std::integral_constant<int, L>{}), ...);
        }(std::make_integer_sequence<int, C::LA + C::LB>{});
    };
    // Point the streams at an item and request its first blocks (the ring must be free).
    auto start_item = [&](const Item& it) {
        if constexpr (KIND != kColsT)
            setup_ptrs<C::A_TRANS, BM, C::NW, C::LA, BK>(it.A, it.lda, it.Mt, wave, lane, pa, ka, g.a_gather, it.row0, g.a_gather_div);
        else
            setup_ptrs<C::A_TRANS, BM, C::NW, C::LA, BK>(it.A, it.lda, it.Mt, wave, lane, pa, ka);
        setup_ptrs<C::B_TRANS, BN, C::NW, C::LB, BK>(it.B, it.ldb, it.Nt, wave, lane, pb, kb);
        stepA = C::A_TRANS ? (long)BK * it.lda : BK;
        stepB = C::B_TRANS ? (long)BK * it.ldb : BK;
#pragma unroll
        for (int l = 0; l < C::LA; ++l) pa[l] += stepA * it.kb0;
#pragma unroll
        for (int l = 0; l < C::LB; ++l) pb[l] += stepB * it.kb0;
        Kt = it.Kt;  kb0 = it.kb0;
        const int nk = it.kb1 - it.kb0;
#pragma unroll
        for (int s = 0; s < STAGES; ++s)
            if (s < nk) issue(s);
    };

    // ---------------- per-lane LDS offsets of the MFMA operand fetches ----------------
    int offA[TM], offB[TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int rb = (wm * TM + i) * 32;
        if constexpr (!C::A_TRANS) {
            offA[i] = (rb + (lane & 31)) * (BK * 2) + ((((lane >> 5)) ^ swz<BK>(lane & 31)) << 4);
        } else {
            const int s = lane & 15, col = rb + ((lane >> 4) & 1) * 16 + 4 * (s & 3);
            offA[i] = ((lane >> 5) * 8 + (s >> 2)) * (BM * 2) + ((swap13(col >> 3) ^ (2 * (s >> 2))) << 4) + (col & 7) * 2;
        }
    }
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int rb = (wn * TN + j) * 32;
        if constexpr (!C::B_TRANS) {
            offB[j] = (rb + (lane & 31)) * (BK * 2) + ((((lane >> 5)) ^ swz<BK>(lane & 31)) << 4);
        } else {
            const int s = lane & 15, col = rb + ((lane >> 4) & 1) * 16 + 4 * (s & 3);
            offB[j] = ((lane >> 5) * 8 + (s >> 2)) * (BN * 2) + ((swap13(col >> 3) ^ (2 * (s >> 2))) << 4) + (col & 7) * 2;
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
    int tm_act = TM;   // 32-row blocks of this wave that hold at least one valid row of the current item

    // Software pipeline over the nk blocks of the current item (its first min(nk, STAGES) blocks have been
    // requested).  Ring slot li % STAGES holds block li.  The operand registers are double-buffered: while the
    // matrix cores work on one 16-deep step, the LDS reads of the next step (which may belong to the next
    // block) are in flight.  Per block there is one barrier, placed after this wave's last LDS read of the
    // block, so that the slot can be refilled right behind it.
    auto main_loop = [&](auto full_tag, const int nk) {
        constexpr bool FULL = decltype(full_tag)::value;
        constexpr int PER = C::LA + C::LB;
        static_assert((BK / 16) % 2 == 0, "even number of MFMA steps per block");
        constexpr int KS = BK / 16;
        bf16x8 fa[2][TM], fb[2][TN];
        auto fetch = [&](int slot, int ks, bf16x8 (&a)[TM], bf16x8 (&b)[TN]) {
            const char* tA = smem + slot * C::STAGE_BYTES;
            const char* tB = tA + C::A_BYTES;
#pragma unroll
            for (int j = 0; j < TN; ++j) b[j] = fetchB(tB, j, ks);
#pragma unroll
            for (int i = 0; i < TM; ++i)
                if (FULL || i < tm_act) a[i] = fetchA(tA, i, ks);
        };
        // One 16-deep MFMA step.  The loads of the block that refills the slot freed at the last barrier are
        // issued during the first step after that barrier, a share before each accumulator row: early, because
        // they have only until the end of this block to arrive.  (Spread evenly over all the block's steps instead,
        // the rows kinds run 3-5 % slower.)
        constexpr int SLOTS = TM;
        auto mma = [&](const bf16x8 (&a)[TM], const bf16x8 (&b)[TN], auto step_c, int load_li) {
            constexpr int STEP = decltype(step_c)::value;
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                if (load_li >= 0) {
                    [&]<int... L>(std::integer_sequence<int, L...>) {
                        ((L * SLOTS / PER == STEP * TM + i ? (issue_one(load_li, std::integral_constant<int, L>{}), 0) : 0), ...);
                    }(std::make_integer_sequence<int, PER>{});
                }
                if (FULL || i < tm_act) {
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
                }
            }
        };
        fetch(0, 0, fa[0], fb[0]);
        int load_li = -1;
        auto steps_before_barrier = [&](int slot) {
            [&]<int... S>(std::integer_sequence<int, S...>) {
                ((fetch(slot, S + 1, fa[(S + 1) & 1], fb[(S + 1) & 1]),
                  mma(fa[S & 1], fb[S & 1], std::integral_constant<int, S + 1>{}, load_li)), ...);
            }(std::make_integer_sequence<int, KS - 1>{});
        };
        for (int li = 0; li + 1 < nk; ++li) {
            steps_before_barrier(li % STAGES);
            // own loads of block li+1 have landed (later blocks may stay in flight) and own LDS reads of
            // block li are complete; after the barrier that holds for every wave
            wait_groups<PER, STAGES - 2>(min(nk - 2 - li, STAGES - 2));
            __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0), other counters untouched
            __builtin_amdgcn_s_barrier();
            load_li = li + STAGES < nk ? li + STAGES : -1;
            fetch((li + 1) % STAGES, 0, fa[0], fb[0]);
            mma(fa[1], fb[1], std::integral_constant<int, 0>{}, load_li);
        }
        steps_before_barrier((nk - 1) % STAGES);   // last block: nothing left to prefetch
        mma(fa[1], fb[1], std::integral_constant<int, 0>{}, -1);
    };

    // ---------------- finishing a work item ----------------
    // Partial sums of a split tile are exchanged through one fp32 buffer per workgroup, in the register layout
    // of the accumulators (thread-major, 16 bytes per thread and accumulator quarter), so a wave-level access is
    // one contiguous kilobyte.  They and the flags are written and read with agent-scope accesses (sc1): these
    // are served where the XCDs' caches meet, so no cache needs to be written back or invalidated, and a store
    // has reached that point when the wave's memory counter has drained.  The reading side lands the buffer in
    // the (idle) LDS ring, many requests in flight at once, and adds it to its accumulators from there.
    typedef __attribute__((ext_vector_type(4))) float f32x4;
    constexpr int PART_ROWS = TM * TN * 4;                       // 16-byte pieces per thread
    constexpr int PART_ROW_BYTES = NT * 16;                      // one piece of every thread
    constexpr int RING_ROWS = C::RING / PART_ROW_BYTES;          // pieces per thread that fit in the ring
    static_assert(RING_ROWS >= 1, "ring too small to land partial sums");
    auto store_partial = [&]() {
        int tid_ = tid;
        asm volatile("" : "+v"(tid_));   // keeps the address arithmetic of this cold path out of the main loop's registers
        char* const dst = (char*)g.sk_part + (size_t)sk_slot * kPartialBytesPerWg + tid_ * 16;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const f32x4 v = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
                    // (the wait states keep the next instruction from overwriting the data registers of a store that
                    // is wider than 64 bits while it still reads them: the compiler inserts them for its own stores
                    // but cannot see into an assembly statement)
                    asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 2"
                                 :: "v"(dst + ((i * TN + j) * 4 + q) * PART_ROW_BYTES), "v"(v) : "memory");
                }
        wait_vmcnt<0>();                       // this wave's partial sums have arrived ...
        __syncthreads();                       // ... and so have those of the other waves
        if (tid == 0) __hip_atomic_store(g.sk_flags + sk_slot, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    };
    // Adds the partial sum of the workgroup just below (same XCD slot, one position lower).  The ring must be idle.
    auto add_predecessor = [&]() {
        const int id = sk_slot - 8;
        if (tid == 0) {
            int spins = 0;
            // (a negative limit gives every wait up at once, flag or no flag: the tests' way to walk through this path)
            while (g.spin_limit < 0 || __hip_atomic_load(g.sk_flags + id, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 1) {
                if (++spins > g.spin_limit) {   // cannot happen (see the header); kept so that every wave ends
                    __hip_atomic_store(g.sk_error, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    break;
                }
                __builtin_amdgcn_s_sleep(16);
            }
            __hip_atomic_store(g.sk_flags + id, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // as the next launch expects
        }
        __syncthreads();
        int tid_ = tid;
        asm volatile("" : "+v"(tid_));
        const char* const src = (const char*)g.sk_part + (size_t)id * kPartialBytesPerWg + tid_ * 16;
        const char* const mine = smem + tid_ * 16;   // every thread reads back exactly what its own wave requested
#pragma unroll
        for (int r0 = 0; r0 < PART_ROWS; r0 += RING_ROWS) {
            // (the waits of this routine are assembly statements with a memory clobber: the compiler must not move
            // the LDS reads across them, which it may do with the plain wait builtin)
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // LDS reads of the previous round are complete
#pragma unroll
            for (int r = r0; r < r0 + RING_ROWS && r < PART_ROWS; ++r)
                asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off sc1"
                             :: "s"(lds_base + (r - r0) * PART_ROW_BYTES + wave * 1024), "v"(src + r * PART_ROW_BYTES) : "memory");
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
            for (int r = r0; r < r0 + RING_ROWS && r < PART_ROWS; ++r) {
                const float4 pz = *(const float4*)(mine + (r - r0) * PART_ROW_BYTES);
                const int i = r / (TN * 4), j = (r / 4) % TN, q = r % 4;
                acc[i][j][4 * q] += pz.x;  acc[i][j][4 * q + 1] += pz.y;
                acc[i][j][4 * q + 2] += pz.z;  acc[i][j][4 * q + 3] += pz.w;
            }
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();              // every wave is done with the ring: the next item's blocks may land
    };
    auto pack8 = [](const float* f) {
        return make_uint4(pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]), pack_bf16x2(f[4], f[5]),
                          pack_bf16x2(f[6], f[7]));
    };
    auto unpack8 = [](const uint4 u, float* f) {
        const unsigned w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            f[2 * t] = __uint_as_float(w[t] << 16);
            f[2 * t + 1] = __uint_as_float(w[t] & 0xffff0000u);
        }
    };
    // Accumulator element v of lane l is row (v/4)*8 + (l/32)*4 + v%4, column l%32 of its 32x32 block: the
    // elements v = 4s .. 4s+3 of a wave's TN blocks form an 8-row slab.  Each wave passes one slab at a time
    // through its private fp32 LDS patch and reads it back row-wise, 8 consecutive columns per lane, so that
    // global memory sees 16-byte pieces of whole rows.  The LDS unit serves a wave's requests in order, so the
    // next slab may be written into the patch as soon as the reads of the current one have been issued; the
    // loop below keeps the patch traffic of slab s+1 and the table look-ups of slab s-1 in flight while the
    // values of slab s are converted and stored.
    constexpr int TNG = C::TNG;                  // accumulator columns per pass through the patch
    constexpr int CPRW = TNG * 4;                // 8-column pieces per row of a column group
    static_assert(8 * CPRW <= 64 && TN % TNG == 0, "a slab of a column group is at most one piece per lane");
    auto epilogue = [&](const Fin& it, auto stream_tag) {
        constexpr bool STREAM = decltype(stream_tag)::value;   // results as streaming stores (GemmArgs::stream_out)
        constexpr bool LOOKUP = C::TABLE;
        const int ldc = g.Nout;
        int lane_ = lane;
        asm volatile("" : "+v"(lane_));   // keeps the address arithmetic of the epilogue out of the main loop's registers
        float* const patch_w = patch + ((lane_ >> 5) * 4) * PITCH + (lane_ & 31);
        const int q = min(lane_, 8 * CPRW - 1);      // (lanes beyond the slab's pieces idle on a copy of the last)
        const int prow = q / CPRW;
        const float* const patch_r = patch + prow * PITCH + (q % CPRW) * 8;
        struct Slab { float4 lo, hi; };
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            if (i >= tm_act) break;
            const int row0 = (wm * TM + i) * 32;
#pragma unroll
            for (int cg = 0; cg < TN / TNG; ++cg) {      // column groups of the wave tile, one after the other
                const int pcol = (wn * TN + cg * TNG) * 32 + (q % CPRW) * 8;
                const bool pok = lane_ < 8 * CPRW && pcol < it.Nt;
                auto to_patch = [&](int sl) {
#pragma unroll
                    for (int j = 0; j < TNG; ++j)
#pragma unroll
                        for (int r = 0; r < 4; ++r) patch_w[r * PITCH + j * 32] = acc[i][cg * TNG + j][4 * sl + r];
                };
                auto from_patch = [&](Slab& v) {
                    v.lo = *(const float4*)patch_r;
                    v.hi = *(const float4*)(patch_r + 4);
                };
                float bias[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};   // of this lane's 8 columns (the same for every row)
                if constexpr (KIND == kRowsNN_GeLU || KIND == kRowsNN) {
                    if (g.bias && pok) unpack8(*(const uint4*)((const u16*)g.bias + it.b_off + pcol), bias);
                }
                uint4 zin[4];
                if constexpr (KIND == kRowsNT_dGeLU) {   // saved pre-activations of the whole block, requested up front
#pragma unroll
                    for (int sl = 0; sl < 4; ++sl) {
                        const int row = row0 + sl * 8 + prow;
                        zin[sl] = make_uint4(0, 0, 0, 0);
                        if (pok && row < it.Mt)
                            zin[sl] = *(const uint4*)((const u16*)g.Zin + it.c_off + (size_t)row * ldc + pcol);
                    }
                }
                Slab cur, nxt;
                float xs[8], fac[8];   // values and looked-up factors of the slab before the current one
                to_patch(0);
                from_patch(cur);
#pragma unroll
                for (int sl = 0; sl <= 4; ++sl) {
                    if (sl + 1 < 4) { to_patch(sl + 1); from_patch(nxt); }
                    if constexpr (LOOKUP) {
                        if (sl > 0) {   // second half of slab sl-1: its factors have arrived
                            const int row = row0 + (sl - 1) * 8 + prow;
                            if (pok && row < it.Mt) {
#pragma unroll
                                for (int t = 0; t < 8; ++t) xs[t] *= fac[t];
                                const size_t o = it.c_off + (size_t)row * ldc + pcol;
                                store_out((uint4*)((u16*)(KIND == kRowsNN_GeLU ? g.C2 : g.C) + o), pack8(xs), STREAM);
                            }
                        }
                    }
                    if (sl == 4) break;
                    const int row = row0 + sl * 8 + prow;
                    if (pok && row < it.Mt) {
                        float x[8] = {cur.lo.x, cur.lo.y, cur.lo.z, cur.lo.w, cur.hi.x, cur.hi.y, cur.hi.z, cur.hi.w};
                        if constexpr (KIND == kRowsNN_GeLU || KIND == kRowsNN) {
#pragma unroll
                            for (int t = 0; t < 8; ++t) x[t] += bias[t];
                        }
                        const size_t o = it.c_off + (size_t)row * ldc + pcol;
                        if constexpr (KIND == kRowsNN_GeLU) {
                            const uint4 zp = pack8(x);
                            store_out((uint4*)((u16*)g.C + o), zp, STREAM);
                            const unsigned w[4] = {zp.x, zp.y, zp.z, zp.w};
#pragma unroll
                            for (int t = 0; t < 4; ++t) {
                                // H = z Phi(z), z in fp32: Phi looked up at the bf16 rounding zb of z, plus the slope
                                // phi(zb) times what the rounding took away (what is left is of second order, 2^-18)
                                const float zlo = __uint_as_float(w[t] << 16), zhi = __uint_as_float(w[t] & 0xffff0000u);
                                // (phi(zb) = 2^(-zb^2 log2(e) / 2) / sqrt(2 pi))
                                fac[2 * t] = fmaf((x[2 * t] - zlo) * 0.39894228040143268f,
                                                  __builtin_amdgcn_exp2f(zlo * zlo * -0.72134752044448170f), act[act_index(w[t])]);
                                fac[2 * t + 1] = fmaf((x[2 * t + 1] - zhi) * 0.39894228040143268f,
                                                      __builtin_amdgcn_exp2f(zhi * zhi * -0.72134752044448170f), act[act_index(w[t] >> 16)]);
                            }
#pragma unroll
                            for (int t = 0; t < 8; ++t) xs[t] = x[t];
                        } else if constexpr (KIND == kRowsNT_dGeLU) {
                            const unsigned w[4] = {zin[sl].x, zin[sl].y, zin[sl].z, zin[sl].w};
#pragma unroll
                            for (int t = 0; t < 4; ++t) {
                                fac[2 * t] = act[act_index(w[t])];
                                fac[2 * t + 1] = act[act_index(w[t] >> 16)];
                            }
#pragma unroll
                            for (int t = 0; t < 8; ++t) xs[t] = x[t];
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
                                    float prev[8];
                                    unpack8(*Ch, prev);
#pragma unroll
                                    for (int t = 0; t < 8; ++t) x[t] += prev[t];
                                }
                                store_out(Ch, pack8(x), STREAM);
                            }
                        } else {
                            size_t oo = o;
                            if constexpr (KIND == kRowsNN) {   // top-1: the row goes straight to its token's place in Y
                                if (g.c_scatter) oo = (size_t)g.c_scatter[it.row0 + row] * ldc + (it.c_off - (size_t)it.row0 * ldc) + pcol;
                            }
                            store_out((uint4*)((u16*)g.C + oo), pack8(x), STREAM);
                        }
                    }
                    cur = nxt;
                }
            }
        }
    };

    // ---------------- the work loop ----------------
    Item cur;
    bool have = next_item(cur);
    if (have) start_item(cur);
    if constexpr (C::TABLE) {
        // built while the first blocks are on their way; visible to all waves after the first barrier, long
        // before the first epilogue (every item of these kinds has at least one block)
        float* w = (float*)(smem + C::RING + C::PATCH_BYTES);
        if (have)
            for (int i = tid; i < 2 * kActEntries; i += NT) w[i] = act_entry<KIND>(i);
    }
    // Number of store instructions a wave issues in the epilogue of a full tile (bf16 output, nothing added to): they
    // are the youngest memory operations when the next item's main loop is about to start, and the memory counter
    // retires in order, so waiting until at most that many operations are outstanding means the item's first blocks
    // (requested before the epilogue) have landed, without waiting for the stores to be acknowledged as well.
    constexpr int kFullTileStores = TM * (TN / C::TNG) * 4 * (KIND == kRowsNN_GeLU ? 2 : 1);
    static_assert(kFullTileStores < 64, "memory counter range");
    bool stores_behind = false;              // the previous item ended with exactly those stores
    while (have) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
        tm_act = (cur.Mt - wm * TM * 32 + 31) / 32;
        tm_act = tm_act < 0 ? 0 : (tm_act > TM ? TM : tm_act);
        const int nk = cur.kb1 - cur.kb0;
        if (nk > 0) {
            // The first blocks of this item were requested before the previous epilogue, whose own memory
            // operations came later: wait for everything but that epilogue's stores (where their number is known),
            // then every wave may read ring slot 0.
            if (stores_behind) wait_vmcnt<kFullTileStores>();
            else wait_vmcnt<0>();
            __builtin_amdgcn_s_barrier();
            if (tm_act == TM) main_loop(std::true_type{}, nk);
            else main_loop(std::false_type{}, nk);   // tail tiles skip the 32-row blocks that hold no valid row
            __builtin_amdgcn_s_waitcnt(0xc07f);
            __builtin_amdgcn_s_barrier();              // every wave is done reading the ring
        }
        const Fin fin{cur.c_off, cur.b_off, cur.Mt, cur.Nt, cur.owner, cur.row0};
        if (cur.kb0 > 0) add_predecessor();   // the blocks before kb0 were summed by the workgroup just below
        have = next_item(cur);
        if (have) start_item(cur);
        if (fin.owner) {
            if (g.stream_out) epilogue(fin, std::true_type{});
            else epilogue(fin, std::false_type{});
        }
        else store_partial();
        stores_behind = fin.owner && fin.Mt == BM && fin.Nt == BN && !(KIND == kColsT && (g.out_f32 || g.accumulate));
    }
    if constexpr (KIND == kColsT) {
        if (dynamic && tid == 0) {       // the last workgroup to finish leaves the counters at zero for the next launch
            const int done = __hip_atomic_fetch_add(g.dyn_counters + 8, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (done == (int)gridDim.x - 1)
                for (int i = 0; i < 9; ++i) __hip_atomic_store(g.dyn_counters + i, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    if (blockIdx.x == 0 && tid == 0) {   // shader cycles and 100 MHz ticks this workgroup lived: the clock the launch ran at
        g.clock_probe[0] = clock64() - probe_cycles0;
        g.clock_probe[1] = wall_clock64() - probe_ticks0;
    }
}

template <int KIND, int WM, int WN, int TM, int TN, int STAGES, int BK>
__global__ __launch_bounds__(WM * WN * 64, 1) void ggemm_sk_kernel(GemmArgs g, int ntm, int ntn)
{
    ggemm_sk_body<KIND, WM, WN, TM, TN, STAGES, BK>(g, ntm, ntn);
}

// The rows of every expert in two size classes, one after the other in one launch: whole blocks of 256 rows in
// 256 x 256 tiles, then the experts' last pieces (at most 128 rows) in 128 x 512 tiles.  The main loop's pace is set by
// the arrival of the operand blocks, not by what a tile holds, so a last piece costs half as much in tiles twice as wide.
// DEEP (chosen by the host for reductions shallower than 2 * kMinSplitDepth, which are never cut into pieces): the
// last pieces in 128 x 128 tiles with 128-deep blocks instead.  A tile's time is its number of blocks times the
// time a block takes to arrive, so the few last pieces, which get a phase of their own behind the big tiles, are
// done in a quarter of the blocks, by four times as many workgroups.
template <int KIND, int STAGES, int BK, bool DEEP>
__device__ __forceinline__ void ggemm_classes(const GemmArgs& g, int ntn_big, int ntn_small)
{
    if constexpr (DEEP) {
        ggemm_sk_body<KIND, 2, 4, 4, 2, STAGES, BK, 1>(g, 0, ntn_big);
        __syncthreads();   // the first class's last epilogue is done with the LDS before the second lays it out anew
        // (only while the narrow tiles are at most one round: beyond that their number counts, not their length, and
        // the wide ones are fewer - measured on a skewed load with 44 last pieces: 7 % slower with the narrow ones)
        const int ntn_deep = (g.Nout + 127) / 128;
        if ((long)g.cls[kClsPSmall * (g.E + 1) + g.E] * ntn_deep <= (long)gridDim.x)
            ggemm_sk_body<KIND, 2, 4, 2, 1, 2, 128, 2>(g, 0, ntn_deep);
        else
            ggemm_sk_body<KIND, 1, 8, 4, 2, 3, 32, 2>(g, 0, ntn_small);
        return;
    }
    const int W = gridDim.x >> 3;
    const long Tb = (long)g.cls[kClsPBig * (g.E + 1) + g.E] * ntn_big, Ts = (long)g.cls[kClsPSmall * (g.E + 1) + g.E] * ntn_small;
    if (g.whole_tiles) {
        // Followed by another product in the same launch: whole tiles only.  The big tiles go round the workgroups
        // from the first on; the last pieces, in 128 x 256 tiles (a 128 x 512 tile of a deep reduction would be the
        // longest item of the launch), start behind the big tiles' last round, so that no workgroup gets one of each.
        ggemm_sk_body<KIND, 2, 4, 4, 2, STAGES, BK, 1>(g, 0, ntn_big);
        if (Ts == 0) return;
        __syncthreads();
        const int after = (int)(((Tb >> 3) + ((Tb & 7) ? 1 : 0)) % W);
        ggemm_sk_body<KIND, 2, 4, 2, 2, 2, 64, 2>(g, 0, ntn_big, after < W - 1 ? after : 0, after < W - 1 ? W - after : W);
        return;
    }
    if (Ts == 0) { ggemm_sk_body<KIND, 2, 4, 4, 2, STAGES, BK, 1>(g, 0, ntn_big); return; }
    if (Tb == 0) { ggemm_sk_body<KIND, 1, 8, 4, 2, 3, 32, 2>(g, 0, ntn_small); return; }
    if (g.K >= 2 * kMinSplitDepth && W >= 2 && Tb < 8L * W) {
        // Deep reductions with less than a round of tiles are cut into equal pieces over the workgroups, so a second
        // phase for the last pieces would leave most workgroups idle: the two classes run side by side instead, on
        // shares of every XCD's workgroups in proportion to their operand bytes (a 128 x 512 tile moves 5/4 of what a
        // 256 x 256 tile moves).  (With whole rounds of tiles the shares would have to match the classes' times more
        // closely than such an estimate can: measured 7 % slower on a large problem.)
        const long cs = Ts * 5, cb = Tb * 4;
        int ws = (int)((W * cs + (cs + cb) / 2) / (cs + cb));
        ws = ws < 1 ? 1 : ws > W - 1 ? W - 1 : ws;
        ggemm_sk_body<KIND, 2, 4, 4, 2, STAGES, BK, 1>(g, 0, ntn_big, 0, W - ws);
        ggemm_sk_body<KIND, 1, 8, 4, 2, 3, 32, 2>(g, 0, ntn_small, W - ws, ws);   // (a workgroup runs one of the two)
        return;
    }
    ggemm_sk_body<KIND, 2, 4, 4, 2, STAGES, BK, 1>(g, 0, ntn_big);
    __syncthreads();   // the first class's last epilogue is done with the LDS before the second lays it out anew
    ggemm_sk_body<KIND, 1, 8, 4, 2, 3, 32, 2>(g, 0, ntn_small);
}

template <int KIND, int STAGES, int BK, bool DEEP>
__global__ __launch_bounds__(512, 1) void ggemm_cls_kernel(GemmArgs g, int ntn_big, int ntn_small)
{
    ggemm_classes<KIND, STAGES, BK, DEEP>(g, ntn_big, ntn_small);
}

// Two products that do not depend on each other in one launch: a rows kind, then the weight gradients with their
// tiles handed out on demand.  A workgroup that runs out of tiles of the first product goes on with the second
// instead of idling until the launch ends, and one launch gap is saved.  CLASSES: the rows kind in size classes
// (as ggemm_cls_kernel), else in 64 x 256 tiles (many small experts).
template <int KIND, bool CLASSES, bool DEEP>
__global__ __launch_bounds__(512, 1) void ggemm_pair_kernel(GemmArgs g1, int ntn1, int ntn1_small, GemmArgs g2, int ntm2, int ntn2)
{
    if constexpr (CLASSES) ggemm_classes<KIND, 2, 64, DEEP>(g1, ntn1, ntn1_small);
    else ggemm_sk_body<KIND, 1, 8, 2, 1, 3, 64>(g1, 0, ntn1);
    __syncthreads();
    ggemm_sk_body<kColsT, 2, 4, 4, 2, 4, 32>(g2, ntm2, ntn2);
}

// Persistent workgroups of one launch: one per compute unit of the current device, a multiple of the 8 XCDs, at most
// kMaxPersistentWgs (the workspace holds one partial-sum buffer per workgroup and phase).  0 after fail_launch.
static int persistent_wgs()
{
    static std::mutex mu;
    static int cached[kMaxDevices] = {};
    const int dev = current_device();
    if (dev < 0) return 0;
    std::lock_guard<std::mutex> lk(mu);
    if (!cached[dev]) {
        int cus = 0;
        const hipError_t e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess) { fail_launch("grouped GEMM: compute-unit count of device %d: %s", dev, hipGetErrorString(e)); return 0; }
        cus = cus / 8 * 8;
        if (cus < 8) { fail_launch("grouped GEMM: device %d has fewer than 8 compute units", dev); return 0; }
        cached[dev] = cus > kMaxPersistentWgs ? kMaxPersistentWgs : cus;
    }
    return cached[dev];
}

template <int KIND, int WM, int WN, int TM, int TN, int STAGES, int BK>
void launch_cfg(const GemmArgs& a, hipStream_t st)
{
    using C = Cfg<KIND, WM, WN, TM, TN, STAGES, BK>;
    static_assert((size_t)C::BM * C::BN * 4 <= kPartialBytesPerWg, "partial-sum buffer");
    auto kern = ggemm_sk_kernel<KIND, WM, WN, TM, TN, STAGES, BK>;
    if (!allow_dynamic_lds(kern, C::SMEM)) return;
    const int wgs = persistent_wgs();
    if (wgs < 8) return;
    const int ntn = (a.Nout + C::BN - 1) / C::BN;
    const int ntm = KIND == kColsT ? (a.K + C::BM - 1) / C::BM : 0;
    hipLaunchKernelGGL(kern, dim3((unsigned)wgs), dim3(C::NT), C::SMEM, st, a, ntm, ntn);
}

template <int KIND> using CfgWide = Cfg<KIND, 1, 8, 4, 2, 3, 32>;
template <int KIND> using CfgDeep = Cfg<KIND, 2, 4, 2, 1, 2, 128>;

template <int KIND, int STAGES, int BK, bool DEEP>
void launch_cls_cfg(const GemmArgs& a, hipStream_t st)
{
    using C1 = Cfg<KIND, 2, 4, 4, 2, STAGES, BK>;
    using C2 = CfgWide<KIND>;
    static_assert((size_t)C2::BM * C2::BN * 4 <= kPartialBytesPerWg, "partial-sum buffer");
    constexpr int SMEM = std::max({C1::SMEM, C2::SMEM, DEEP ? CfgDeep<KIND>::SMEM : 0});
    auto kern = ggemm_cls_kernel<KIND, STAGES, BK, DEEP>;
    if (!allow_dynamic_lds(kern, SMEM)) return;
    const int wgs = persistent_wgs();
    if (wgs < 8) return;
    hipLaunchKernelGGL(kern, dim3((unsigned)wgs), dim3(512), SMEM, st, a, (a.Nout + C1::BN - 1) / C1::BN,
                       (a.Nout + C2::BN - 1) / C2::BN);
}

template <int KIND, int STAGES, int BK>
void launch_cls(const GemmArgs& a, hipStream_t st)
{
    if (a.K < 2 * kMinSplitDepth) launch_cls_cfg<KIND, STAGES, BK, true>(a, st);
    else launch_cls_cfg<KIND, STAGES, BK, false>(a, st);
}

template <int KIND> void launch_kind(const GemmArgs& a, hipStream_t st)
{
    // 256 x 256 tile, 8 waves of 128 x 64, and a 128 KB ring: two slots of 64-deep blocks, or four slots of 32-deep
    // blocks.  The finer ring keeps three quarters of itself in flight instead of half, which hides more of the
    // operands' latency, at the price of twice as many barriers; measured, it is 5 % faster for the weight gradients
    // and for FC2, even for FC1 and dXs, and 10 % slower for dH, so each kind gets its better one.
    // (Two workgroups of 4 waves per compute unit, each on a 256 x 128 tile with 32-deep blocks, so that one computes
    // while the other waits or writes its tile, are 15-20 % slower: they move half as much again into LDS per flop.)
    // Many small experts (fewer than 96 rows on average): 64 x 256 tiles, 8 waves of 64 x 32, 3 ring slots, so that a
    // tile is not mostly rows that do not exist.  (The weight gradients keep the large tile: their tile spans the
    // weight matrix, not the expert's rows.)
    // Otherwise the rows kinds run in two size classes (launch_cls): an expert's last few rows in 128 x 512 tiles.
    if constexpr (KIND != kColsT) {
        if (a.M < 96L * a.E) { launch_cfg<KIND, 1, 8, 2, 1, 3, 64>(a, st); return; }
        if (!a.cls) { fail_launch("grouped GEMM: the plan step's size-class tables are missing"); return; }
        if constexpr (KIND == kRowsNN) launch_cls<KIND, 4, 32>(a, st);
        else launch_cls<KIND, 2, 64>(a, st);
    } else {
        launch_cfg<KIND, 2, 4, 4, 2, 4, 32>(a, st);
    }
}
}  // namespace sk

namespace sk {
template <int KIND, bool CLASSES, bool DEEP>
void launch_pair_cfg(const GemmArgs& rows, const GemmArgs& cols, hipStream_t st)
{
    using C1 = std::conditional_t<CLASSES, Cfg<KIND, 2, 4, 4, 2, 2, 64>, Cfg<KIND, 1, 8, 2, 1, 3, 64>>;
    using C1s = CfgWide<KIND>;
    using C2 = Cfg<kColsT, 2, 4, 4, 2, 4, 32>;
    constexpr int SMEM = std::max({C1::SMEM, CLASSES ? C1s::SMEM : 0, CLASSES && DEEP ? CfgDeep<KIND>::SMEM : 0, C2::SMEM});
    auto kern = ggemm_pair_kernel<KIND, CLASSES, DEEP>;
    if (!allow_dynamic_lds(kern, SMEM)) return;
    const int wgs = persistent_wgs();
    if (wgs < 8) return;
    GemmArgs r = rows, c = cols;
    c.on_demand = 1;
    r.whole_tiles = 1;
    const int ntn1 = (r.Nout + C1::BN - 1) / C1::BN, ntn1s = (r.Nout + C1s::BN - 1) / C1s::BN;
    const int ntn2 = (c.Nout + C2::BN - 1) / C2::BN, ntm2 = (c.K + C2::BM - 1) / C2::BM;
    hipLaunchKernelGGL(kern, dim3((unsigned)wgs), dim3(512), SMEM, st, r, ntn1, ntn1s, c, ntm2, ntn2);
}

template <int KIND> void launch_pair_kind(const GemmArgs& rows, const GemmArgs& cols, hipStream_t st)
{
    if (rows.M < 96L * rows.E) launch_pair_cfg<KIND, false, false>(rows, cols, st);   // as in launch_kind
    else if (rows.K < 2 * kMinSplitDepth) launch_pair_cfg<KIND, true, true>(rows, cols, st);
    else launch_pair_cfg<KIND, true, false>(rows, cols, st);
}
}  // namespace sk

// With few tiles per workgroup the ragged end of a rows-kind launch (a quarter to half a tile per workgroup) and the
// launch gap are worth more than the counter's round trips; measured, the pair wins up to about 8 tiles per
// workgroup (C1: -3 % per step, C2: -1.4 %) and loses 0.5 % at 34 (C4).
// How often a workgroup polls for its predecessor's partial sum before it gives up and sets the workspace's status
// word.  MOE355_SPIN_LIMIT overrides the default (about a second); a negative value makes every wait give up at once,
// which is how the tests reach the status word without making anything hang.
static int spin_limit()
{
    const char* s = getenv("MOE355_SPIN_LIMIT");
    return s && *s ? atoi(s) : sk::kSpinLimit;
}

bool ggemm_pair_pays(const GemmArgs& rows)
{
    const int wgs = sk::persistent_wgs();
    if (wgs < 8) return false;
    const long row_tiles = rows.M / 256 + rows.E / 2, col_tiles = (rows.Nout + 255) / 256;
    return row_tiles * col_tiles <= 8L * wgs;
}

void launch_ggemm_pair_bf16_sk(const GemmArgs& rows_, const GemmArgs& cols_, hipStream_t st)
{
    using namespace sk;
    GemmArgs rows = rows_, cols = cols_;
    rows.spin_limit = cols.spin_limit = spin_limit();
    if (rows.kind == kRowsNT_dGeLU) launch_pair_kind<kRowsNT_dGeLU>(rows, cols, st);
    else launch_pair_kind<kRowsNT>(rows, cols, st);
}

void launch_ggemm_bf16_sk(const GemmArgs& a_, hipStream_t st)
{
    using namespace sk;
    GemmArgs a = a_;
    a.spin_limit = spin_limit();
    switch (a.kind) {
        case kRowsNN_GeLU: launch_kind<kRowsNN_GeLU>(a, st); break;
        case kRowsNN: launch_kind<kRowsNN>(a, st); break;
        case kRowsNT_dGeLU: launch_kind<kRowsNT_dGeLU>(a, st); break;
        case kRowsNT: launch_kind<kRowsNT>(a, st); break;
        default: launch_kind<kColsT>(a, st); break;
    }
}

}  // namespace moe
