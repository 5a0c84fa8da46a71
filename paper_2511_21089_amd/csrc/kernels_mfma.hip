// Prefill path: bf16 MFMA kernels for gfx950 (v_mfma_f32_16x16x32_bf16, wave64).
//
// Kernel 1  gate_up_mfma:  H[t,j] = bf16( alpha_b(j) * SiLU(<x_t,Wg_j>) * <x_t,Wu_j> )
//           one tile of tokens x neurons per workgroup with TWO fp32 accumulator sets (gate and
//           up), so the gated product of Sec. 3.1's inner bracket is formed in registers and
//           only H (bf16) leaves the CU.
// Kernel 2  down_mfma:     out[t,m] = sum_{j in active runs} H[t,j] * Wd[m,j]
//           one tile of tokens x output features per workgroup; the K loop walks every active
//           run back to back, so the sum over branches of Sec. 3.1 is one fp32 accumulation with
//           no per-branch round trip.  Small outputs are split along K into partial sums that a
//           second kernel adds up in a fixed order.
//
// Both kernels share one main loop: BMT A rows (tokens) against two blocks of 32 NB B rows, waves in
// a WM x 2 arrangement, each wave owning (BMT / WM) x (16 NB + 16 NB) outputs as 16x16 MFMA tiles.
// Tile shapes in use: 256 x (128 + 128) and 256 x (64 + 64) with 8 waves and the whole LDS of a CU,
// 128 x (64 + 64) with 4 waves and either half the LDS (two workgroups per CU) or a deeper ring,
// 64 x (64 + 64) with 4 waves and a ring of whole K tiles (five requested ahead).  The
// 16x16x32 shape is used rather than 32x32x16 because the chip is power limited on this work: with
// random operands a pure stream of 16x16x32 MFMAs sustains 2.0 PFLOP/s, one of 32x32x16 1.7.
#include <algorithm>

#include "internal.h"

namespace mlpmoe {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int BM = 256;          // tokens per tile of the large-tile kernels (and of the routed path's tables)
constexpr int BM_SMALL = 128;    // tokens per tile of the small-tile kernels
constexpr int BNH_MAX = 128;     // rows of each of the two B blocks: 32 * NB, NB = 4 (128) or 2 (64)
constexpr int BK = 64;           // K elements per tile: one tile row is 128 bytes = one cache line
// The LDS is a ring that keeps the K tile in use and the D tiles requested ahead of it.  Two layouts:
//   alternating (the 256-token tiles): 2 D + 1 parts of equal size, A0 B0 A1 B1 A2 | B2 A3 ...; with D = 2 the
//       ring fills the LDS of a CU (five parts of 32 KiB), half a K tile less than whole stages would need;
//   staged: D + 1 stages, a stage being the A rows followed by the B rows of one K tile.  Nothing is padded, so
//       tiles with fewer A rows than B rows keep more K tiles in flight in the same LDS.
__host__ __device__ constexpr int n_parts(int depth) { return 2 * depth + 1; }
// A part of the alternating ring holds the A rows (BMT tokens), or the B rows (2 blocks of 32 NB), of one K tile.
// 256-token tiles: 32 KiB parts, the ring is the whole LDS of a CU (one workgroup of 8 waves per CU).
// 128-token tiles with NB = 2: 16 KiB parts, 80 KiB per workgroup of 4 waves, two workgroups per CU.
__host__ __device__ constexpr int part_bytes(int bmt, int nb) { return (bmt > 64 * nb ? bmt : 64 * nb) * BK * 2; }
__host__ __device__ constexpr int stage_bytes(int bmt, int nb) { return (bmt + 64 * nb) * BK * 2; }
__host__ __device__ constexpr int lds_bytes(int bmt, int nb, int depth = 2, bool staged = false)
{
    return staged ? (depth + 1) * stage_bytes(bmt, nb) : n_parts(depth) * part_bytes(bmt, nb);
}
constexpr int MFMA_WM = 4;                           // waves along M of the 256-token tiles: 8 waves of 64 x (64+64) outputs
constexpr int SMALL_WM = 2;                          // ... of the 128-token tiles: 4 waves of 64 x (32+32)
constexpr int BM_SLIM = 64;                          // tokens per tile of the slim kernels: 4 waves of 32 x (32+32)
constexpr int SLIM_WM = 2;

enum { DST_F32 = 0, DST_BF16 = 1 };     // how down_mfma writes its result

// 16 zero bytes: K chunks that fall past the end of a range are fetched from here.
__device__ const uint32_t g_zero_chunk[4] = {0, 0, 0, 0};

typedef const __attribute__((address_space(1))) void *gptr_t;
typedef __attribute__((address_space(3))) void *lptr_t;

// One wave-wide 16-byte-per-lane load straight into LDS: lane l's data lands at dst + 16*l.
__device__ __forceinline__ void dma16(const void *src, void *lds_dst)
{
    __builtin_amdgcn_global_load_lds((gptr_t)src, (lptr_t)lds_dst, 16, 0, 0);
}

// Workgroup barrier that waits until at most N of this wave's direct-to-LDS loads (they return
// in issue order) and none of its LDS reads are outstanding.  Written by hand because the
// compiler's own barrier waits for every load, which would drain the multi-stage pipeline.
template <int N>
__device__ __forceinline__ void pipeline_barrier()
{
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory");
    __builtin_amdgcn_sched_barrier(0);
}

// Position in the flattened list of K tiles (ranges laid end to end).
struct KCursor {
    int run, k;
};

// K ranges of the gate/up projection: the whole model dimension.
struct KSingle {
    int len;
    __device__ __forceinline__ int n_runs() const { return 1; }
    __device__ __forceinline__ int start(int) const { return 0; }
    __device__ __forceinline__ int end(int) const { return len; }
};
// K ranges of the down projection: the active runs of neurons.
struct KRuns {
    const BranchTable &bt;
    __device__ __forceinline__ int n_runs() const { return bt.n_runs; }
    __device__ __forceinline__ int start(int r) const { return bt.run_start[r]; }
    __device__ __forceinline__ int end(int r) const { return bt.run_end[r]; }
};

// K ranges chosen per workgroup at run time (per-token routing: the branches some token of this
// token tile is routed to).  Lane r of every wave holds the bounds of range r; reading them is a
// lane read, not a memory access.
struct KRunsLanes {
    int n, v_start, v_end;
    __device__ __forceinline__ int n_runs() const { return n; }
    __device__ __forceinline__ int start(int r) const { return __builtin_amdgcn_readlane(v_start, r); }
    __device__ __forceinline__ int end(int r) const { return __builtin_amdgcn_readlane(v_end, r); }
};

// Merged ranges of the branches that are active AND flagged in `needed` (B bytes, uniform).
__device__ __forceinline__ KRunsLanes routed_runs(const BranchTable &bt, const uint8_t *needed)
{
    KRunsLanes kr{0, 0, 0};
    const int lane = threadIdx.x & 63;
    int prev_end = -1;
    for (int b = 0; b < bt.B; ++b) {
        if (!((bt.active >> b) & 1ULL) || !needed[b]) continue;
        const int s = bt.off[b], e = bt.off[b + 1];
        if (e == s) continue;
        if (kr.n > 0 && prev_end == s) {
            kr.v_end = lane == kr.n - 1 ? e : kr.v_end;
        } else {
            kr.v_start = lane == kr.n ? s : kr.v_start;
            kr.v_end = lane == kr.n ? e : kr.v_end;
            ++kr.n;
        }
        prev_end = e;
    }
    return kr;
}

template <typename KR>
__device__ __forceinline__ KCursor k_seek(const KR &kr, int tile)
{
    KCursor c{0, 0};
    for (int r = 0; r < kr.n_runs(); ++r) {
        const int n = (kr.end(r) - kr.start(r) + BK - 1) / BK;
        if (tile < n) {
            c.run = r;
            c.k = kr.start(r) + tile * BK;
            return c;
        }
        tile -= n;
    }
    c.run = kr.n_runs() - 1;
    c.k = kr.start(c.run);
    return c;
}

// LDS layout.  The LDS is a ring of 2 D + 1 parts (five parts of 32 KiB for the 256-token tiles).  A part
// holds rows of 128 bytes (8 chunks of 8 bf16): either the A rows (tokens) of one K tile, or its B rows (the
// rows of the first B block, then those of the second).  Parts are filled in the order A0 B0 A1 B1 A2 B2 ...,
// part number s going to ring slot s % (2 D + 1), so while K tile i is being used the parts of tiles i+1 ..
// i+D-1 and the A part of tile i+D are landing.  Chunk c of row r is stored at chunk slot c ^ swz(r),
// swz(r) = (r & 7) ^ ((r >> 3) & 1), so that the 16-byte reads of 32 consecutive rows at one
// logical chunk (and of 16 consecutive rows at 4 consecutive chunks) fall on distinct banks.  A direct-to-LDS wave load writes 1 KiB = 8 whole rows,
// and each row is one full 128-byte line of global memory (half lines cost the same L2 -> CU
// transfer as whole ones); the swizzle is applied on the global side: the lane that fills slot p
// of row r fetches logical chunk p ^ swz(r).
//
// Main loop, WM x 2 waves.  A_tile / B0_tile / B1_tile point at the first row of the tile (wave uniform);
// a_valid / b0_valid / b1_valid are the rows that exist from there on (>= 1).  Rows past that
// are clamped to the last valid row: their results are never stored and MFMA rows / columns do
// not mix.  K chunks past the end of a range are read from a zero chunk, in A and in B.
// Schedule of K tile i (two K steps of 32; fragments are double buffered one step ahead):
//   step 0: MFMAs; read step 1's fragments; issue the A part of tile i+D
//   barrier: parts of tile i+1 have landed (only the loads issued after them may be in flight) and
//            every wave has read its last fragments of tile i, whose two ring slots are free again
//   step 1: MFMAs; read step 0's fragments of tile i+1; issue the B part of tile i+D
// The direct loads are spread over the steps (one per wave every other MFMA slot) because a
// CU's vector memory path takes about as long to move a tile as the MFMAs take to consume it:
// issued in bursts, the loads back up in the issue queue and the MFMAs behind them wait.
// NB = 16-row MFMA pieces per B block per wave: 4 (B blocks of 128 rows, a 256 x 256 tile) or 2 (B
// blocks of 64 rows, a 256 x 128 tile, for shapes that would otherwise leave most CUs without a
// tile in the last round).  A B part of 64 + 64 rows fills half of its ring slot.
template <int BMT, int WM, int NB, int D, bool kStaged, bool kRowsAreB, typename KR>
__device__ __forceinline__ void mainloop(const uint16_t *__restrict__ A_tile, int lda, int a_valid,
                                         const uint16_t *__restrict__ B0_tile,
                                         const uint16_t *__restrict__ B1_tile, int ldb, int b0_valid,
                                         int b1_valid, const KR &kr, int kt_begin, int kt_end, char *lds,
                                         f32x4 (&acc0)[BMT / 16 / WM][NB], f32x4 (&acc1)[BMT / 16 / WM][NB])
{
    constexpr int MI = BMT / 16 / WM;             // 16-row MFMA tiles per wave along M
    constexpr int NWAVES = WM * 2;
    constexpr int BNH = 32 * NB;                  // rows of each B block
    constexpr int PL = BMT / 8 / NWAVES;          // 1 KiB wave-loads per wave per A part
    constexpr int PLB = 8 * NB / NWAVES;          // ... per B part
    constexpr int N_SLOTS = MI * NB / 2;          // slots of 4 MFMAs per K step
    constexpr int N_PIECES = 2 * NB + MI;         // fragment pieces per K step
    constexpr int RPS = (N_PIECES + N_SLOTS - 1) / N_SLOTS < 2 ? 2 : (N_PIECES + N_SLOTS - 1) / N_SLOTS;   // fragment reads per slot
    // Ring geometry in bytes: where the A part of the first K tile and its B part sit, how far the next tile's
    // parts are from this tile's, and where the ring wraps.
    // direct loads of a part, spread over the slots of a K step: every *_EVERY-th slot issues *_PER of them
    constexpr int A_EVERY = PL <= N_SLOTS ? N_SLOTS / PL : 1, A_PER = PL <= N_SLOTS ? 1 : PL / N_SLOTS;
    constexpr int B_EVERY = PLB <= N_SLOTS ? N_SLOTS / PLB : 1, B_PER = PLB <= N_SLOTS ? 1 : PLB / N_SLOTS;
    constexpr int B_FIRST = kStaged ? BMT * 128 : part_bytes(BMT, NB);
    constexpr int RING_STEP = kStaged ? stage_bytes(BMT, NB) : 2 * part_bytes(BMT, NB);
    constexpr int RING_BYTES = lds_bytes(BMT, NB, D, kStaged);
    static_assert(D >= 2, "one tile in use, at least one more on its way");
    static_assert((N_SLOTS % PL == 0 || PL % N_SLOTS == 0) && (N_SLOTS % PLB == 0 || PLB % N_SLOTS == 0) &&
                      PL % 2 == 0 && PLB % 2 == 0,
                  "loads spread evenly over the slots, slab parity is load parity");
    const int nk = kt_end - kt_begin;
    if (nk <= 0) return;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;

    // ---- global side: per-lane byte offsets of this wave's loads, relative to the tile pointers
    const int lr = lane >> 3;                     // row inside the 8-row slab of one wave-load
    const int cl0 = (lane & 7) ^ lr;              // logical chunk fetched in even slabs; odd slabs: cl0 ^ 1
    const bool second = wave >= NWAVES / 2;       // this wave fills the rows of the second B block
    const int b_valid = second ? b1_valid : b0_valid;
    unsigned a_off[PL], b_off[PLB];
#pragma unroll
    for (int n = 0; n < PL; ++n) {
        const int slab = wave * PL + n;
        const int cl = cl0 ^ (n & 1);             // PL is even, so slab parity is n parity
        int ra = slab * 8 + lr;
        ra = ra < a_valid ? ra : a_valid - 1;
        a_off[n] = (unsigned)ra * (unsigned)lda * 2u + (unsigned)cl * 16u;
    }
#pragma unroll
    for (int n = 0; n < PLB; ++n) {
        const int slab = wave * PLB + n;          // 0 .. 8 NB - 1; the second half are B1's rows
        const int cl = cl0 ^ (n & 1);
        int rb = (slab % (4 * NB)) * 8 + lr;
        rb = rb < b_valid ? rb : b_valid - 1;
        b_off[n] = (unsigned)rb * (unsigned)ldb * 2u + (unsigned)cl * 16u;
    }
    const char *a_base = reinterpret_cast<const char *>(A_tile);
    const char *b_base = reinterpret_cast<const char *>(second ? B1_tile : B0_tile);
    char *wa_dst = lds + wave * (PL * 1024);      // this wave's slabs inside an A part
    char *wb_dst = lds + wave * (PLB * 1024);     // ... inside a B part
    const char *zero = reinterpret_cast<const char *>(g_zero_chunk);

    // Position of the next part to be issued, per matrix.  `left` counts the tiles not yet
    // issued.  A lane whose chunk lies past the end of the K range, or any lane once no tile is
    // left, reads the zero chunk instead.  Branch free, so that the loads sit in the same basic
    // block as the MFMAs and every part is always the same number of loads.
    struct Issue {
        int run, k, kend, left, off;              // off: byte offset in the ring of the part to be filled next
    };
    auto advance = [&](Issue &q) {                // stays on the last range once the list is exhausted
        q.k += BK;
        if (q.k >= q.kend && q.run + 1 < kr.n_runs()) {
            ++q.run;
            q.k = kr.start(q.run);
            q.kend = kr.end(q.run);
        }
        --q.left;
        q.off += RING_STEP;
        if (q.off >= RING_BYTES) q.off -= RING_BYTES;
    };
    // what the loads of one part have in common
    struct Part {
        const char *src;                          // tile pointer moved to the part's K offset
        char *dst;                                // this wave's first slab in the part's ring slot
        bool ok[2];                               // chunk inside the K range, for even / odd slabs
    };
    auto part_of = [&](const Issue &q, const char *base, char *w_dst) {
        Part pt;
        const int kend = q.left > 0 ? q.kend : -(1 << 30);
        pt.src = base + (size_t)q.k * 2;
        pt.dst = w_dst + q.off;
        pt.ok[0] = q.k + cl0 * 8 < kend;
        pt.ok[1] = q.k + (cl0 ^ 1) * 8 < kend;
        return pt;
    };
    auto dma_part = [&](int n, const Part &pt, const unsigned *off) {
        dma16(pt.ok[n & 1] ? pt.src + off[n] : zero, pt.dst + n * 1024);
    };

    // ---- LDS side: per-lane read offsets (bytes) for the 2 K steps of a tile.  A 16x16x32
    // fragment is 16 rows x 32 K: lane l holds row l & 15 and K group l >> 4 (8 elements).  Which
    // 16-byte chunk of the step's 64 bytes a K group reads is free as long as A and B agree (the
    // dot product does not care about the order of K).  The LDS serves lanes l and l + 32 in the
    // same cycle, so K groups g and g + 2 are given ADJACENT chunks (0, 2, 1, 3 -> chunks 0, 1, 2,
    // 3): with the row swizzle the 16 lanes of a cycle then fall on distinct banks.
    const int lrow = lane & 15;
    const int swz = (lane & 7) ^ ((lane >> 3) & 1);      // fragment rows start at multiples of 16
    const int kg = lane >> 4;
    const int kchunk = ((kg & 1) << 1) | (kg >> 1);
    int a_rd[2], b_rd[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
        const int slot = (ks * 4 + kchunk) ^ swz;
        a_rd[ks] = (wm * (MI * 16) + lrow) * 128 + slot * 16;
        b_rd[ks] = (wn * (16 * NB) + lrow) * 128 + slot * 16;
    }
    // Fragment pieces of one K step: v[0 .. 2 NB) = the B pieces b0[0..NB), b1[0..NB) (16 rows of the
    // first / second B block each), then the A pieces.  MFMA m uses A piece m / (2 NB) and B piece
    // m % (2 NB).
    struct Frags {
        bf16x8 v[N_PIECES];
    };
    auto read_piece = [&](Frags &f, int g, int a_at, int ks) {
        // the B part of a tile follows its A part (alternating ring: in the next part, which may be the first)
        const int b_at = kStaged ? a_at + B_FIRST : (a_at + B_FIRST < RING_BYTES ? a_at + B_FIRST : 0);
        if (g < 2 * NB)
            f.v[g] = *reinterpret_cast<const bf16x8 *>(lds + b_at + b_rd[ks] + (g / NB) * (BNH * 128) +
                                                       (g % NB) * (16 * 128));
        else
            f.v[g] = *reinterpret_cast<const bf16x8 *>(lds + a_at + a_rd[ks] + (g - 2 * NB) * (16 * 128));
    };
    // kRowsAreB: the B rows (weights) are the MFMA's row operand and the A rows (tokens) its column
    // operand.  In the 16x16 result lane l then holds column l & 15 = one token and rows
    // 4 * (l >> 4) + 0..3 = four consecutive B rows, which the epilogues store as one 8- or 16-byte
    // piece of the token's output row.  Otherwise tokens are the rows.
    auto mfma_n = [&](const Frags &f, int m) {
        const int i = m / (2 * NB), b = m % (2 * NB);
        const bf16x8 r = kRowsAreB ? f.v[b] : f.v[2 * NB + i], c = kRowsAreB ? f.v[2 * NB + i] : f.v[b];
        if (b < NB) acc0[i][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(r, c, acc0[i][b], 0, 0, 0);
        else acc1[i][b - NB] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(r, c, acc1[i][b - NB], 0, 0, 0);
    };
    // One K step, written in the instruction order wanted: slots of {4 MFMAs, then LDS reads of
    // the next step's fragments, then (in evenly spaced slots) one direct load}; nothing may be
    // moved across a slot boundary.  The compiler waits for ALL outstanding LDS reads before the
    // first MFMA of a step (direct-to-LDS loads in flight make it give up exact counting), so the
    // reads are packed into the early slots and the last slots leave them time to land.
    // DMA: 1 loads of the A part pt, 2 loads of the B part pt.
    auto k_step = [&](const Frags &cur_f, Frags &nxt_f, int rd_at, int rd_ks, int dma, const Part &pt) {
#pragma unroll
        for (int g = 0; g < N_SLOTS; ++g) {
            // The two waves of a SIMD take the matrix pipe in turns of four MFMAs.  A wave asks
            // for its turn at priority 1 (first MFMA), holds it at priority 3 (the other wave,
            // asking at 1, cannot cut in, which the older wave otherwise always does) and drops
            // to 0 for its loads and address arithmetic, which then run under the other's turn.
            __builtin_amdgcn_s_setprio(1);
            mfma_n(cur_f, 4 * g);
            __builtin_amdgcn_s_setprio(3);
#pragma unroll
            for (int q = 1; q < 4; ++q) mfma_n(cur_f, 4 * g + q);
            __builtin_amdgcn_s_setprio(0);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int r = 0; r < RPS; ++r)
                if (RPS * g + r < N_PIECES) read_piece(nxt_f, RPS * g + r, rd_at, rd_ks);
            if (dma == 1 && g % A_EVERY == 0) {
#pragma unroll
                for (int l = 0; l < A_PER; ++l) dma_part((g / A_EVERY) * A_PER + l, pt, a_off);
            }
            if (dma == 2 && g % B_EVERY == 0) {
#pragma unroll
                for (int l = 0; l < B_PER; ++l) dma_part((g / B_EVERY) * B_PER + l, pt, b_off);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // prologue: the parts of tiles 0 .. D-1 in flight, tile 0 landed
    Issue qa, qb;
    {
        const KCursor c = k_seek(kr, kt_begin);
        qa.run = c.run;
        qa.k = c.k;
        qa.kend = kr.end(c.run);
        qa.left = nk;
        qa.off = 0;
        qb = qa;
        qb.off = B_FIRST;
    }
#pragma unroll
    for (int p = 0; p < D; ++p) {
        const Part pa = part_of(qa, a_base, wa_dst), pb = part_of(qb, b_base, wb_dst);
#pragma unroll
        for (int n = 0; n < PL; ++n) dma_part(n, pa, a_off);
#pragma unroll
        for (int n = 0; n < PLB; ++n) dma_part(n, pb, b_off);
        advance(qa);
        advance(qb);
    }
    pipeline_barrier<(D - 1) * (PL + PLB)>();
    Frags f0, f1;
#pragma unroll
    for (int g = 0; g < N_PIECES; ++g) read_piece(f0, g, 0, 0);

    int rd = 0;                                   // byte offset in the ring of the A part of the tile in use
    for (int it = 0; it < nk; ++it) {
        const Part pa = part_of(qa, a_base, wa_dst);
        k_step(f0, f1, rd, 1, 1, pa);             // + A part of tile it+D
        advance(qa);
        // tile it+1 has landed (the newer tiles and the A part just issued may be in flight); tile it's slots are free
        pipeline_barrier<(D - 2) * (PL + PLB) + PL>();
        rd = rd + RING_STEP < RING_BYTES ? rd + RING_STEP : rd + RING_STEP - RING_BYTES;
        const Part pb = part_of(qb, b_base, wb_dst);
        k_step(f1, f0, rd, 0, 2, pb);             // + B part of tile it+D
        advance(qb);
    }
    pipeline_barrier<0>();                        // LDS may be reused by the caller
}

__device__ __forceinline__ int branch_of(const BranchTable &bt, int j)
{
    int b = 0;
    while (b + 1 < bt.B && j >= bt.off[b + 1]) ++b;
    return b;
}

__device__ __forceinline__ float silu_mul(float g, float u)
{
    // SiLU(g) * u with hardware exp2 / rcp (about 1 ulp each)
    const float e = __builtin_amdgcn_exp2f(g * -1.4426950408889634f);
    return g * __builtin_amdgcn_rcpf(1.0f + e) * u;
}

__device__ __forceinline__ uint16_t to_bf16(float v)
{
    const __bf16 b = (__bf16)v;          // v_cvt_pk_bf16_f32: round to nearest even
    return __builtin_bit_cast(uint16_t, b);
}

// Workgroup id -> output tile.  The hardware deals consecutive workgroup ids round-robin to the
// 8 XCDs, each with its own L2.  Every XCD therefore takes one contiguous eighth of a "grouped"
// tile order (groups of 8 M tiles, M fastest inside a group), so that the 32 workgroups resident
// on an XCD form an 8 x 4 block of tiles and share their A and B tiles through that L2.
// The grid holds 8 * ceil(tiles / 8) ids; ids past the end get no tile.
constexpr int XCDS = 8;
constexpr int GROUP_M = 8;
__host__ __device__ inline int ids_per_xcd(long long tiles) { return (int)((tiles + XCDS - 1) / XCDS); }
// position in the grouped tile order -> tile
__device__ __forceinline__ void tile_from_logical(int logical, int tiles_m, int tiles_n, int &tm, int &tn)
{
    const int group_sz = GROUP_M * tiles_n;
    const int g = logical / group_sz, rem = logical % group_sz;
    const int m0 = g * GROUP_M;
    const int gsz = tiles_m - m0 < GROUP_M ? tiles_m - m0 : GROUP_M;
    tm = m0 + rem % gsz;
    tn = rem / gsz;
}
__device__ __forceinline__ bool tile_of(int id, int tiles_m, int tiles_n, int &tm, int &tn)
{
    const int total = tiles_m * tiles_n;
    const int logical = (id % XCDS) * ids_per_xcd(total) + id / XCDS;
    if (logical >= total) return false;
    const int group_sz = GROUP_M * tiles_n;
    const int g = logical / group_sz, rem = logical % group_sz;
    const int m0 = g * GROUP_M;
    const int gsz = tiles_m - m0 < GROUP_M ? tiles_m - m0 : GROUP_M;
    tm = m0 + rem % gsz;
    tn = rem / gsz;
    return true;
}

// Scratch of the routed kernels, filled by route_tile_list from route[T, B]:
//   tile_need[tm * B + b]  != 0 if some token of token tile tm (256 tokens) is routed to branch b;
//   counts[g], list[g * stride + i]: the live gate+up tiles of token-tile group g (GROUP_M token
//   tiles) in the order the kernel walks them: by N tile, then by token tile.  An entry is
//   tn * gsz + (tm - g * GROUP_M), gsz = token tiles in the group.  A tile is live if some token of
//   its token tile is routed to an active branch that owns one of its neurons.
struct RouteTiles {
    const uint8_t *tile_need;
    const uint32_t *counts;
    const uint32_t *list;
    int stride;
};

// N tile tn (counted over the runs of active branches, tiles of bnh neurons) -> its first neuron and
// the end of its run; false past the last tile.
__device__ __forceinline__ bool neuron_tile(const BranchTable &bt, int tn, int bnh, int &n0, int &n_end)
{
    for (int r = 0; r < bt.n_runs; ++r) {
        const int n = (bt.run_end[r] - bt.run_start[r] + bnh - 1) / bnh;
        if (tn < n) {
            n0 = bt.run_start[r] + tn * bnh;
            n_end = bt.run_end[r];
            return true;
        }
        tn -= n;
    }
    return false;
}

// One tile of the gate+up projection: tokens tm * BMT .., neurons n0 .. min(n0 + 32 NB, n_end) of a run that
// ends at n_end.  lds: lds_bytes(BMT, NB, D) bytes.
template <int BMT, int WM, int NB, int D, bool kStaged, bool kRouted>
__device__ __forceinline__ void gate_up_tile(const uint16_t *__restrict__ X, const uint16_t *__restrict__ Wg,
                                             const uint16_t *__restrict__ Wu, uint16_t *__restrict__ H, int T,
                                             int d_model, int ldh, const uint8_t *__restrict__ route,
                                             const BranchTable &bt, char *lds, int tm, int n0, int n_end)
{
    constexpr int BNH = 32 * NB;
    const int t0 = tm * BMT;

    constexpr int MI = BMT / 16 / WM;
    f32x4 accg[MI][NB], accu[MI][NB];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            accg[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
            accu[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
        }

    const int nk = (d_model + BK - 1) / BK;
    mainloop<BMT, WM, NB, D, kStaged, true>(X + (size_t)t0 * d_model, d_model, T - t0, Wg + (size_t)n0 * d_model,
                       Wu + (size_t)n0 * d_model, d_model, n_end - n0, n_end - n0, KSingle{d_model}, 0, nk,
                       lds, accg, accu);

    // alpha of the tile's neurons -> LDS (the main loop is done with it)
    float *al = reinterpret_cast<float *>(lds);
    int *bl = reinterpret_cast<int *>(lds + BNH_MAX * sizeof(float));      // branch of each neuron (routing)
    if (threadIdx.x < BNH) {
        const int n = n0 + threadIdx.x;
        const int b = branch_of(bt, n < n_end ? n : n_end - 1);
        al[threadIdx.x] = n < n_end ? bt.alpha[b] : 0.f;
        if (kRouted) bl[threadIdx.x] = b;
    }
    __syncthreads();

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int tcol = lane & 15, q4 = lane >> 4;
#pragma unroll
    for (int i = 0; i < MI; ++i) {
        const int t = t0 + wm * (MI * 16) + i * 16 + tcol;
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            const int nl = wn * (16 * NB) + j * 16 + 4 * q4;   // first of 4 neurons, tile relative
            // run ends are multiples of 8: the four neurons are all inside the run or all outside
            if (t < T && n0 + nl < n_end) {
                const f32x4 a4 = *reinterpret_cast<const f32x4 *>(al + nl);
                uint16_t h[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    float v = a4[q] * silu_mul(accg[i][j][q], accu[i][j][q]);
                    if (kRouted) v = route[(size_t)t * bt.B + bl[nl + q]] ? v : 0.f;
                    h[q] = to_bf16(v);
                }
                u32x2 pk;
                pk.x = (uint32_t)h[0] | ((uint32_t)h[1] << 16);
                pk.y = (uint32_t)h[2] | ((uint32_t)h[3] << 16);
                *reinterpret_cast<u32x2 *>(H + (size_t)t * ldh + n0 + nl) = pk;
            }
        }
    }
}

// grid.x = 8 * ids_per_xcd(tilesM * sum over runs of N tiles).
// kRouted: per-token routing.  route[t * B + b] != 0 says token t takes branch b.  Only the live
// tiles are computed: workgroup ids are dealt over the compacted tile list as tile_of() deals them
// over the full grid (one contiguous stretch of the list per XCD), the ids left over exit.  The
// down projection skips the same (token tile, branch) pairs, and H is multiplied by the token's
// route bit, so that it is exactly 0 where a token does not take a branch.
template <int BMT, int WM, int NB, int D, bool kStaged, bool kRouted>
__global__ void __launch_bounds__(WM * 128)
gate_up_mfma(const uint16_t *__restrict__ X, const uint16_t *__restrict__ Wg,
             const uint16_t *__restrict__ Wu, uint16_t *__restrict__ H, int T, int d_model, int d_inter,
             int ldh, int tiles_m, int tiles_n, const uint8_t *__restrict__ route, RouteTiles rt,
             BranchTable bt)
{
    static_assert(!kRouted || BMT == BM, "the routed path's tables are per 256 tokens");
    __shared__ __attribute__((aligned(1024))) char lds[lds_bytes(BMT, NB, D, kStaged)];
    constexpr int BNH = 32 * NB;                  // neurons per tile
    int tm, tn;
    if (kRouted) {
        const int groups = (tiles_m + GROUP_M - 1) / GROUP_M;
        int total = 0;
        for (int g = 0; g < groups; ++g) total += (int)rt.counts[g];
        const int per_xcd = ids_per_xcd(total);
        const int k = blockIdx.x / XCDS;
        const int logical = (blockIdx.x % XCDS) * per_xcd + k;
        if (k >= per_xcd || logical >= total) return;
        int g = 0, before = 0;
        for (; g < groups - 1; ++g) {
            const int c = (int)rt.counts[g];
            if (logical < before + c) break;
            before += c;
        }
        const int e = (int)rt.list[(size_t)g * rt.stride + (logical - before)];
        const int m0 = g * GROUP_M;
        const int gsz = tiles_m - m0 < GROUP_M ? tiles_m - m0 : GROUP_M;
        tm = m0 + e % gsz;
        tn = e / gsz;
    } else if (!tile_of(blockIdx.x, tiles_m, tiles_n, tm, tn)) {
        return;
    }
    int n0, n_end;
    if (!neuron_tile(bt, tn, BNH, n0, n_end)) return;
    gate_up_tile<BMT, WM, NB, D, kStaged, kRouted>(X, Wg, Wu, H, T, d_model, ldh, route, bt, lds, tm, n0, n_end);
}

// The gate+up projection with WIDE tiles for the full rounds of 256 workgroups and smaller tiles for what
// is left, when that is at most half a round: the left-over wide tiles, cut into REST pieces, then fill one
// (shorter) round instead of leaving more than half of the CUs idle for a wide one.  REST = 2: halves of
// 64 neurons (NARROW's tile); REST = 4, when at most a quarter of a round is left: quarters of 128 tokens x
// 64 neurons, run by the same eight waves as 32 x (32 + 32) outputs each.
// Workgroup ids below 8 * wide_per_xcd take wide tiles: id i is tile (i % 8) * P + i / 8 of the grouped
// order, P = ids_per_xcd(wide tiles), i.e. every XCD works through the first wide_per_xcd tiles of its
// contiguous eighth.  The ids above take the rest of each eighth, REST consecutive ids per wide tile (the
// neuron half alternates fastest).  grid.x = 8 * (wide_per_xcd + REST * (P - wide_per_xcd)).
constexpr int QUARTER_D = 3;                          // ring depth of the quarter tiles (7 parts of 16 KiB)
template <int WM, int REST>
__global__ void __launch_bounds__(WM * 128)
gate_up_mfma_mixed(const uint16_t *__restrict__ X, const uint16_t *__restrict__ Wg,
                   const uint16_t *__restrict__ Wu, uint16_t *__restrict__ H, int T, int d_model, int ldh,
                   int tiles_m, int tiles_n, int wide_per_xcd, BranchTable bt)
{
    static_assert(REST == 2 || REST == 4, "halves or quarters of a wide tile");
    static_assert(lds_bytes(BM / 2, 2, QUARTER_D) <= lds_bytes(BM, 4), "the quarter tiles' ring fits the wide tiles' LDS");
    __shared__ __attribute__((aligned(1024))) char lds[lds_bytes(BM, 4)];
    const int total = tiles_m * tiles_n;
    const int P = ids_per_xcd(total);
    const int xcd = blockIdx.x % XCDS;
    const int xcd_end = (xcd + 1) * P < total ? (xcd + 1) * P : total;
    int k = blockIdx.x / XCDS;
    int tm, tn, n0, n_end;
    if (k < wide_per_xcd) {
        const int logical = xcd * P + k;
        if (logical >= xcd_end) return;
        tile_from_logical(logical, tiles_m, tiles_n, tm, tn);
        if (!neuron_tile(bt, tn, 128, n0, n_end)) return;
        gate_up_tile<BM, WM, 4, 2, false, false>(X, Wg, Wu, H, T, d_model, ldh, nullptr, bt, lds, tm, n0, n_end);
    } else {
        k -= wide_per_xcd;
        const int logical = xcd * P + wide_per_xcd + k / REST;
        if (logical >= xcd_end) return;
        tile_from_logical(logical, tiles_m, tiles_n, tm, tn);
        if (!neuron_tile(bt, tn, 128, n0, n_end)) return;
        n0 += (k % 2) * 64;
        if (n0 >= n_end) return;                                   // the run ends in the first half
        if (REST == 2) {
            gate_up_tile<BM, WM, 2, 2, false, false>(X, Wg, Wu, H, T, d_model, ldh, nullptr, bt, lds, tm, n0, n_end);
        } else {
            const int tq = 2 * tm + (k % 4) / 2;                   // token tile of 128
            if (tq * (BM / 2) >= T) return;                        // the last token tile ends in its first half
            gate_up_tile<BM / 2, WM, 2, QUARTER_D, false, false>(X, Wg, Wu, H, T, d_model, ldh, nullptr, bt, lds, tq,
                                                                 n0, n_end);
        }
    }
}

// grid.x = 8 * ids_per_xcd(splits * tilesM * tilesN); dst = out (splits == 1) or partial[split][T][d_model].
// dst_mode: DST_F32 plain float stores; DST_BF16 (only with splits == 1) dst holds bf16 values, each sum
// rounded once (RNE).
// kRouted: the K loop of token tile tm walks only the branches some token of the tile is routed
// to (tile_need); H is 0 for the tokens of the tile that do not take a branch.
template <int BMT, int WM, int NB, int D, bool kStaged, bool kRouted>
__global__ void __launch_bounds__(WM * 128)
down_mfma(const uint16_t *__restrict__ H, const uint16_t *__restrict__ Wd, float *__restrict__ dst, int T,
          int d_model, int d_inter, int ldh, int tiles_m, int tiles_n, int splits, int kt_total, int dst_mode,
          const uint8_t *__restrict__ tile_need, BranchTable bt)
{
    static_assert(!kRouted || BMT == BM, "the routed path's tables are per 256 tokens");
    __shared__ __attribute__((aligned(1024))) char lds[lds_bytes(BMT, NB, D, kStaged)];
    // Work items are (split, tile in the grouped order), split slowest, and every XCD takes one contiguous
    // eighth of that list: with K split, an XCD then works on few splits, whose slices of H and W_down are
    // what its L2 has to hold (the 0.5B-shaped layer at T = 2048: 4.7 MB per XCD instead of 12.5 MB).
    const int tiles = tiles_m * tiles_n;
    const long long items = (long long)tiles * splits;
    const int per_xcd = ids_per_xcd(items);
    const long long item = (long long)(blockIdx.x % XCDS) * per_xcd + blockIdx.x / XCDS;
    if (item >= items) return;
    const int z = (int)(item / tiles);
    int tm, tn;
    tile_from_logical((int)(item % tiles), tiles_m, tiles_n, tm, tn);
    constexpr int BNH = 32 * NB;                  // output features per B block; a tile has two
    const int t0 = tm * BMT, n0 = tn * (2 * BNH);
    KRunsLanes dyn{0, 0, 0};
    if (kRouted) {
        dyn = routed_runs(bt, tile_need + (size_t)tm * bt.B);
        kt_total = 0;
        for (int r = 0; r < dyn.n; ++r) kt_total += (dyn.end(r) - dyn.start(r) + BK - 1) / BK;
    }
    const int kt_begin = (int)((long long)kt_total * z / splits);
    const int kt_end = (int)((long long)kt_total * (z + 1) / splits);

    constexpr int MI = BMT / 16 / WM;
    f32x4 acc0[MI][NB], acc1[MI][NB];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            acc0[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
            acc1[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
        }

    // the second block of output features may start past d_model: point it at the last row
    const int n1 = n0 + BNH < d_model ? n0 + BNH : d_model - 1;
    if (kRouted)
        mainloop<BMT, WM, NB, D, kStaged, true>(H + (size_t)t0 * ldh, ldh, T - t0, Wd + (size_t)n0 * d_inter,
                                    Wd + (size_t)n1 * d_inter, d_inter, d_model - n0, d_model - n1, dyn, kt_begin,
                                    kt_end, lds, acc0, acc1);
    else
        mainloop<BMT, WM, NB, D, kStaged, true>(H + (size_t)t0 * ldh, ldh, T - t0, Wd + (size_t)n0 * d_inter,
                                    Wd + (size_t)n1 * d_inter, d_inter, d_model - n0, d_model - n1, KRuns{bt},
                                    kt_begin, kt_end, lds, acc0, acc1);

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int tcol = lane & 15, q4 = lane >> 4;
    float *o = dst + (size_t)z * T * d_model;
#pragma unroll
    for (int i = 0; i < MI; ++i) {
        const int t = t0 + wm * (MI * 16) + i * 16 + tcol;
#pragma unroll
        for (int half = 0; half < 2; ++half)
#pragma unroll
            for (int j = 0; j < NB; ++j) {
                const int m = n0 + half * BNH + wn * (16 * NB) + j * 16 + 4 * q4;
                // d_model is a multiple of 8: the four features are all inside or all outside
                if (t < T && m < d_model) {
                    const f32x4 v = half ? acc1[i][j] : acc0[i][j];
                    if (dst_mode == DST_BF16) {
                        u32x2 pk;
                        pk.x = (uint32_t)to_bf16(v[0]) | ((uint32_t)to_bf16(v[1]) << 16);
                        pk.y = (uint32_t)to_bf16(v[2]) | ((uint32_t)to_bf16(v[3]) << 16);
                        *reinterpret_cast<u32x2 *>(reinterpret_cast<uint16_t *>(dst) + (size_t)t * d_model + m) = pk;
                    } else {
                        *reinterpret_cast<f32x4 *>(o + (size_t)t * d_model + m) = v;
                    }
                }
            }
    }
}

constexpr int ROUTE_MAX_TILES_N = 32768;           // N tiles of the gate+up projection the tile list handles

// Fills the routed kernels' scratch (see RouteTiles) for one group of GROUP_M token tiles per
// workgroup.  BNH = neurons per gate+up tile; tiles_n = N tiles over the runs of active branches.
template <int BNH>
__global__ void __launch_bounds__(1024)
route_tile_list(const uint8_t *__restrict__ route, uint8_t *__restrict__ tile_need, uint32_t *__restrict__ counts,
                uint32_t *__restrict__ list, int stride, int T, int tiles_m, int tiles_n, BranchTable bt)
{
    __shared__ uint8_t need[GROUP_M][MLPMOE_MAX_BRANCHES];
    __shared__ uint8_t live[ROUTE_MAX_TILES_N];
    __shared__ int s_off[MLPMOE_MAX_BRANCHES + 1], s_run_start[MLPMOE_MAX_BRANCHES], s_run_end[MLPMOE_MAX_BRANCHES];
    __shared__ int wave_sum[16];
    const int B = bt.B;
    const int g = blockIdx.x, m0 = g * GROUP_M;
    const int gsz = tiles_m - m0 < GROUP_M ? tiles_m - m0 : GROUP_M;
    for (int i = threadIdx.x; i < GROUP_M * MLPMOE_MAX_BRANCHES; i += 1024) (&need[0][0])[i] = 0;
    if (threadIdx.x < 64) {
        // branch table -> LDS: constant indices keep the reads of the kernel arguments scalar
        const int l = threadIdx.x;
        int v_off = 0, v_start = 0, v_end = 0;
#pragma unroll
        for (int i = 0; i < MLPMOE_MAX_BRANCHES; ++i) v_off = l == i ? bt.off[i] : v_off;
#pragma unroll
        for (int i = 0; i < kMaxRuns; ++i) {
            v_start = l == i ? bt.run_start[i] : v_start;
            v_end = l == i ? bt.run_end[i] : v_end;
        }
        s_off[l] = v_off;
        s_run_start[l] = v_start;
        s_run_end[l] = v_end;
        if (l == 0) s_off[MLPMOE_MAX_BRANCHES] = bt.off[MLPMOE_MAX_BRANCHES];
    }
    __syncthreads();
    // the group's rows of route are one contiguous stretch of bytes.  Flags already set are not
    // stored again: the LDS serialises the lanes of a store to one address, reads are broadcast
    const size_t base = (size_t)m0 * BM * B;
    const long long t_end = (long long)(m0 + gsz) * BM < T ? (long long)(m0 + gsz) * BM : T;
    const int n_bytes = (int)((t_end - (long long)m0 * BM) * B);
    const uint8_t *rg = route + base;
    // 16 bytes at a time where the pointer allows it, several loads in flight per thread; one
    // division per 16 bytes, the (token, branch) of the following bytes by stepping
    const int n_vec = (reinterpret_cast<uintptr_t>(rg) & 15u) == 0 ? n_bytes / 16 : 0;
    for (int c0 = threadIdx.x; c0 < n_vec; c0 += 4 * 1024) {
        u32x4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int c = c0 + u * 1024;
            v[u] = c < n_vec ? *reinterpret_cast<const u32x4 *>(rg + (size_t)c * 16) : u32x4{0, 0, 0, 0};
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if ((v[u][0] | v[u][1] | v[u][2] | v[u][3]) == 0) continue;
            const int i = (c0 + u * 1024) * 16;
            int t = i / B, b = i - t * B;
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                if (((v[u][k / 4] >> (8 * (k % 4))) & 0xffu) && !need[t / BM][b]) need[t / BM][b] = 1;
                if (++b == B) {
                    b = 0;
                    ++t;
                }
            }
        }
    }
    for (int i0 = n_vec * 16 + threadIdx.x; i0 < n_bytes; i0 += 8 * 1024) {
        uint8_t v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int i = i0 + u * 1024;
            v[u] = i < n_bytes ? rg[i] : (uint8_t)0;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (v[u]) {
                const int i = i0 + u * 1024;
                if (!need[(i / B) / BM][i % B]) need[(i / B) / BM][i % B] = 1;
            }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < gsz * B; i += 1024) tile_need[(size_t)m0 * B + i] = need[i / B][i % B];

    // live[tn]: bit j says tile (m0 + j, tn) is live; one thread per N tile.  The branch table was
    // copied to LDS above, so that the walks over runs and branches are chains of LDS reads.
    for (int tn = threadIdx.x; tn < tiles_n; tn += 1024) {
        int n0 = 0, n1 = 0, left = tn;
        bool found = false;
        for (int r = 0; r < bt.n_runs; ++r) {
            const int n = (s_run_end[r] - s_run_start[r] + BNH - 1) / BNH;
            if (!found && left < n) {
                n0 = s_run_start[r] + left * BNH;
                n1 = n0 + BNH < s_run_end[r] ? n0 + BNH : s_run_end[r];
                found = true;
            }
            left -= n;
        }
        unsigned bits = 0;
        for (int b = 0; b < B; ++b) {
            const int lo = s_off[b], hi = s_off[b + 1];
            if (!((bt.active >> b) & 1ULL) || hi <= lo || hi <= n0 || lo >= n1) continue;   // owns no neuron of the tile
            for (int j = 0; j < GROUP_M; ++j) bits |= need[j][b] ? 1u << j : 0u;
        }
        live[tn] = (uint8_t)bits;
    }
    __syncthreads();

    // compaction in list order (by N tile, then token tile): every thread takes a contiguous stretch
    // of N tiles, an exclusive prefix over the threads gives its first position
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int per = (tiles_n + 1023) / 1024;
    const int tn0 = threadIdx.x * per;
    const int tn1 = tn0 + per < tiles_n ? tn0 + per : tiles_n;
    int mine = 0;
    for (int tn = tn0; tn < tn1; ++tn) mine += __popc((unsigned)live[tn]);
    int incl = mine;
    for (int d = 1; d < 64; d <<= 1) {
        const int v = __shfl_up(incl, d);
        incl += lane >= d ? v : 0;
    }
    if (lane == 63) wave_sum[wave] = incl;
    __syncthreads();
    int pos = incl - mine, total = 0;
    for (int w = 0; w < 16; ++w) {
        pos += w < wave ? wave_sum[w] : 0;
        total += wave_sum[w];
    }
    if (threadIdx.x == 0) counts[g] = (uint32_t)total;
    for (int tn = tn0; tn < tn1; ++tn)
        for (int j = 0; j < gsz; ++j)
            if ((live[tn] >> j) & 1) list[(size_t)g * stride + pos++] = (uint32_t)(tn * gsz + j);
}

// out[i] = sum_z partial[z][i], summed in z order: deterministic.  out_bf16: out holds bf16 values.
// n4 = pieces of four values (T * d_model is a multiple of 8 on this path; partial is 256-byte, out 16-byte
// aligned).  Two pieces per thread and trip, so that 2 * splits loads are in flight per thread.
__global__ void __launch_bounds__(256)
reduce_partials(const float *__restrict__ partial, float *__restrict__ out, size_t n4, int splits, int out_bf16)
{
    const f32x4 *p4 = reinterpret_cast<const f32x4 *>(partial);
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n4; i += 2 * stride) {
        const size_t j = i + stride;
        const bool two = j < n4;
        f32x4 s0 = p4[i], s1 = two ? p4[j] : f32x4{0.f, 0.f, 0.f, 0.f};
        for (int z = 1; z < splits; ++z) {
            const f32x4 a = p4[(size_t)z * n4 + i];
            const f32x4 b = two ? p4[(size_t)z * n4 + j] : f32x4{0.f, 0.f, 0.f, 0.f};
            s0 += a;
            s1 += b;
        }
        if (out_bf16) {
            u32x2 *o = reinterpret_cast<u32x2 *>(out);
            u32x2 pk;
            pk.x = (uint32_t)to_bf16(s0[0]) | ((uint32_t)to_bf16(s0[1]) << 16);
            pk.y = (uint32_t)to_bf16(s0[2]) | ((uint32_t)to_bf16(s0[3]) << 16);
            o[i] = pk;
            if (two) {
                pk.x = (uint32_t)to_bf16(s1[0]) | ((uint32_t)to_bf16(s1[1]) << 16);
                pk.y = (uint32_t)to_bf16(s1[2]) | ((uint32_t)to_bf16(s1[3]) << 16);
                o[j] = pk;
            }
        } else {
            f32x4 *o = reinterpret_cast<f32x4 *>(out);
            o[i] = s0;
            if (two) o[j] = s1;
        }
    }
}

int k_tiles(const BranchTable &bt)
{
    int n = 0;
    for (int r = 0; r < bt.n_runs; ++r) n += ceil_div(bt.run_end[r] - bt.run_start[r], BK);
    return n;
}

// Tile shapes.  WIDE: 256 tokens x (128 + 128) rows of B, the shape with the most reuse per byte moved
// into the LDS.  NARROW: 256 x (64 + 64).  SMALL: 128 x (64 + 64) with 4 waves and 80 KiB of LDS, two
// workgroups per CU: four times the tiles of WIDE, the fixed cost of one workgroup (first loads,
// epilogue, hand-over) hidden under the main loop of the other, at 1.6 times WIDE's traffic into the
// LDS per flop.  For layers and batches that give WIDE too few or too short tiles.
// MIXED (gate+up only): WIDE for the full rounds of 256 workgroups, NARROW for a last round that WIDE tiles
// would fill less than half; quarters of a wide tile (128 tokens x (64 + 64)) where they fit one round.
// DEEP: SMALL's tile with four K tiles requested ahead instead of two (a ring of 9 parts, 144 KiB, one
// workgroup per CU): for batches of a few dozen to a hundred tokens, where a launch has about one tile per
// CU and is bound by how many bytes of weights it keeps in flight, not by the matrix cores.
// SLIM: 64 tokens x (64 + 64) with 4 waves and a staged ring of five K tiles requested ahead (144 KiB, one
// workgroup per CU): the A rows of a K tile take a third of a stage, so more bytes of the B operand are in
// flight per CU than with any other shape; for outputs with few token rows per output feature (a down
// projection with a short d_model can then do without a K split) and for batches of at most 64 tokens.
enum TileShape { TILE_WIDE = 0, TILE_NARROW = 1, TILE_SMALL = 2, TILE_MIXED = 3, TILE_DEEP = 4, TILE_SLIM = 5 };
constexpr int N_TILE_SHAPES = 6;
constexpr int DEEP_D = 4, SLIM_D = 5;
// compile-time side of a tile shape: tokens, waves along M, 16-row MFMA pieces per B block and wave, K tiles
// requested ahead, ring layout
template <int BMT_, int WM_, int NB_, int D_, bool kStaged_>
struct ShapeT {
    static constexpr int BMT = BMT_, WM = WM_, NB = NB_, D = D_;
    static constexpr bool kStaged = kStaged_;
};
using ShapeWide = ShapeT<BM, MFMA_WM, 4, 2, false>;
using ShapeNarrow = ShapeT<BM, MFMA_WM, 2, 2, false>;
using ShapeSmall = ShapeT<BM_SMALL, SMALL_WM, 2, 2, false>;
using ShapeDeep = ShapeT<BM_SMALL, SMALL_WM, 2, DEEP_D, false>;
using ShapeSlim = ShapeT<BM_SLIM, SLIM_WM, 2, SLIM_D, true>;
struct TileDims {
    int bm, bn;       // tokens, B rows per block (a tile has two blocks)
    int per_cu;       // workgroups resident per CU
};
constexpr TileDims kTileDims[N_TILE_SHAPES] = {{BM, 128, 1}, {BM, 64, 1}, {BM_SMALL, 64, 2}, {BM, 128, 1}, {BM_SMALL, 64, 1},
                                               {BM_SLIM, 64, 1}};
constexpr int kCUs = 256;

long long gate_up_tiles(const BranchTable &bt, int T, TileShape sh)
{
    long long n = 0;
    for (int r = 0; r < bt.n_runs; ++r) n += ceil_div(bt.run_end[r] - bt.run_start[r], kTileDims[sh].bn);
    return n * ceil_div(T, kTileDims[sh].bm);
}

// Estimated duration in microseconds of a launch of `tiles` tiles with nk K tiles each that streams
// `bytes` of weights and activations, fitted to measurements on the two benchmark layers (T = 64 .. 4096):
// a K tile of a WIDE tile takes about 1.48 us at the clocks the chip sustains on this work, a NARROW one
// 0.62 of that, a SMALL one 0.4 (two share a CU, each at a quarter of a WIDE tile's flops but bound by the
// traffic into the LDS; an odd one at the end runs alone at about 0.3); the fixed cost of a workgroup
// (first loads, epilogue, hand-over) is about 7.4 / 5.2 us and 1.5 us for SMALL, whose neighbour on the CU
// computes meanwhile; DEEP (SMALL's tile alone on its CU) 0.75 and 4.4 us; SLIM 0.6 and 3.5 us.  A launch that
// has few tiles per CU cannot stream faster than about 3.5 TB/s, 5 TB/s with DEEP's and SLIM's longer queues of
// requests.
constexpr double kDeepStreamBytesPerUs = 5.0e6;
double launch_cost_us(long long tiles, int nk, TileShape sh, double bytes)
{
    static const double per_k[N_TILE_SHAPES] = {1.48, 0.92, 0.59, 1.48, 0.75, 0.6}, fixed[N_TILE_SHAPES] = {7.4, 5.2, 1.5, 7.4, 4.4, 3.5};
    const long long per_cu = (tiles + kCUs - 1) / kCUs;       // tiles the busiest CU runs, one after the other
    double c;
    if (sh == TILE_SMALL)
        c = (double)(per_cu / 2) * 2 * (nk * per_k[sh] + fixed[sh]) + (double)(per_cu % 2) * (nk * 0.44 + 4.4);
    else
        c = (double)per_cu * (nk * per_k[sh] + fixed[sh]);
    // DEEP keeps twice the bytes in flight
    return std::max(c, bytes / (sh == TILE_DEEP || sh == TILE_SLIM ? kDeepStreamBytesPerUs : 3.5e6) + fixed[sh]);
}

// Wide tiles that MIXED runs as wide, per XCD (32 per full round of 256), or -1 if MIXED does not apply:
// it needs at least one full round and a remainder of at most half a round.
int mixed_wide_per_xcd(long long wide_tiles)
{
    const long long rounds = wide_tiles / kCUs, rest = wide_tiles % kCUs;
    if (rounds < 1 || rest == 0 || rest > kCUs / 2 || wide_tiles > 0x3fffffffLL) return -1;
    return (int)(rounds * (kCUs / XCDS));
}

// Pieces MIXED cuts each left-over wide tile into: quarters when they fit one round, else halves.
int mixed_rest_parts(long long wide_tiles) { return wide_tiles % kCUs <= kCUs / 4 ? 4 : 2; }

TileShape pick_gate_up_tile(const BranchTable &bt, int T, int d_model)
{
    const int nk = ceil_div(d_model, BK);
    const double bytes = 4.0 * bt.d_eff * d_model;            // W_gate and W_up rows of the active neurons, once
    const long long wide = gate_up_tiles(bt, T, TILE_WIDE);
    TileShape best = TILE_WIDE;
    double best_cost = launch_cost_us(wide, nk, TILE_WIDE, bytes);
    for (TileShape sh : {TILE_NARROW, TILE_SMALL, TILE_DEEP, TILE_SLIM}) {
        if (sh == TILE_SLIM && T > BM_SLIM) continue;           // more tokens: a taller tile reuses the weights
        const double c = launch_cost_us(gate_up_tiles(bt, T, sh), nk, sh, bytes);
        if (c < best_cost * 0.97) {
            best = sh;
            best_cost = c;
        }
    }
    if (mixed_wide_per_xcd(wide) >= 0) {
        // the full rounds as wide tiles, then one round of narrow ones, or of quarters (measured 2 us shorter
        // at 14 K tiles)
        const double c = launch_cost_us(wide / kCUs * kCUs, nk, TILE_WIDE, 0.0) + launch_cost_us(kCUs, nk, TILE_NARROW, 0.0) -
                         (mixed_rest_parts(wide) == 4 ? 2.0 : 0.0);
        if (c < best_cost * 0.97) best = TILE_MIXED;
    }
    return best;
}

// Split-K factor of the down projection: fills the chip when the output has few tiles.
int down_splits(int T, int d_model, int k_elems, TileShape sh)
{
    const TileDims &d = kTileDims[sh];
    const long long tiles = (long long)ceil_div(T, d.bm) * ceil_div(d_model, 2 * d.bn);
    const int kt = ceil_div(k_elems > 0 ? k_elems : 1, BK);
    long long s = (long long)kCUs * d.per_cu / tiles;
    if (s > kt / 4) s = kt / 4;
    if (s > 32) s = 32;
    return s < 1 ? 1 : (int)s;
}

// How the down projection of one call is launched: tile shape and K split (the partial results of a split
// go through the workspace and a second kernel adds them up in a fixed order; adding two halves into
// the result with float atomics instead was measured 2.4 times slower on the 0.5B-shaped layer).
struct DownPlan {
    TileShape shape;
    int splits;
};

DownPlan plan_down(const FwdArgs &a, const BranchTable &bt, bool routed)
{
    const int kt = std::max(1, k_tiles(bt));
    DownPlan best{TILE_WIDE, 1};
    double best_cost = 1e30;
    for (TileShape sh : {TILE_WIDE, TILE_NARROW, TILE_SMALL, TILE_DEEP, TILE_SLIM}) {
        if (a.tile_shape >= 0 && a.tile_shape != (int)TILE_MIXED && a.tile_shape != (int)sh) continue;
        if (routed && kTileDims[sh].bm != BM) continue;
        const TileDims &d = kTileDims[sh];
        const long long tiles = (long long)ceil_div(a.T, d.bm) * ceil_div(a.d_model, 2 * d.bn);
        int sp = std::min(down_splits(a.T, a.d_model, bt.d_eff, sh), kt);
        if (sp > 1 && (size_t)sp * a.T * a.d_model * sizeof(float) > a.partial_bytes) sp = 1;
        // split as far as it fills the chip; the second kernel that adds the sp partial sums up costs about
        // 6 us plus (sp + 1) * T * d_model floats at 8 TB/s
        double c = launch_cost_us(tiles * sp, ceil_div(kt, sp), sh, 2.0 * bt.d_eff * (a.d_model + a.T));
        if (sp > 1) c += 6.0 + (sp + 1.0) * (double)a.T * a.d_model * 4.0 / 8e6;
        if (c < best_cost) {
            best = DownPlan{sh, sp};
            best_cost = c;
        }
    }
    return best;
}

}  // namespace

int mfma_down_splits(int T, int d_model, int k_elems) { return down_splits(T, d_model, k_elems, TILE_WIDE); }

// Layout of the routed kernels' scratch block (256-byte aligned): tile_need, counts, list.
// The list holds, per group of GROUP_M token tiles, up to GROUP_M * (N tiles) entries; the N tiles
// over runs of active branches number at most d_inter / 128 + one per run.
namespace {
int route_list_stride(int d_inter) { return GROUP_M * (d_inter / BNH_MAX + MLPMOE_MAX_BRANCHES + 1); }
size_t route_need_bytes(int T) { return align_up((size_t)ceil_div(T, BM) * MLPMOE_MAX_BRANCHES, 256); }
size_t route_counts_bytes(int T) { return align_up((size_t)ceil_div(ceil_div(T, BM), GROUP_M) * sizeof(uint32_t), 256); }
}  // namespace

size_t route_scratch_bytes(int T, int d_inter)
{
    if (T < 1) T = 1;
    if (d_inter < 0) d_inter = 0;
    const size_t groups = (size_t)ceil_div(ceil_div(T, BM), GROUP_M);
    return route_need_bytes(T) + route_counts_bytes(T) +
           align_up(groups * route_list_stride(d_inter) * sizeof(uint32_t), 256);
}

size_t mfma_partial_bytes(int T, int d_model, int d_inter)
{
    // the largest any tile shape asks for
    int s = 1;
    for (TileShape sh : {TILE_WIDE, TILE_NARROW, TILE_SMALL, TILE_DEEP, TILE_SLIM}) s = std::max(s, down_splits(T, d_model, d_inter, sh));
    return s > 1 ? align_up((size_t)s * T * d_model * sizeof(float), 256) : 0;
}

template <typename S, bool kRouted = false>
static hipError_t launch_gate_up(const FwdArgs &a, const BranchTable &bt)
{
    constexpr int BMT = S::BMT, WM = S::WM, NB = S::NB;
    const int tiles_m = ceil_div(a.T, BMT);
    long long tiles_n = 0;
    for (int r = 0; r < bt.n_runs; ++r) tiles_n += ceil_div(bt.run_end[r] - bt.run_start[r], 32 * NB);
    const long long grid = (long long)XCDS * ids_per_xcd(tiles_m * tiles_n);
    if (grid > 0x7fffffffLL) return note_hip_error("gate_up_mfma grid", hipErrorInvalidValue);
    RouteTiles rt{nullptr, nullptr, nullptr, 0};
    if (kRouted) {
        // one launch builds the tile list (and tile_need, which the down projection reads as well)
        static_assert(!kRouted || 32 * NB == BNH_MAX, "the list's row stride is sized for wide tiles");
        uint8_t *need = a.route_scratch;
        uint32_t *counts = reinterpret_cast<uint32_t *>(a.route_scratch + route_need_bytes(a.T));
        uint32_t *list = reinterpret_cast<uint32_t *>(a.route_scratch + route_need_bytes(a.T) + route_counts_bytes(a.T));
        const int stride = route_list_stride(a.d_inter);
        if ((long long)GROUP_M * tiles_n > stride || tiles_n > ROUTE_MAX_TILES_N)
            return note_hip_error("route tile list size", hipErrorInvalidValue);
        {
            ProfileScope ps(MLPMOE_KERNEL_ROUTE_TILES, a.stream);
            route_tile_list<32 * NB><<<ceil_div(tiles_m, GROUP_M), 1024, 0, a.stream>>>(
                a.route, need, counts, list, stride, a.T, tiles_m, (int)tiles_n, bt);
        }
        if (launch_status("route_tile_list launch") != hipSuccess) return hipErrorLaunchFailure;
        rt = RouteTiles{need, counts, list, stride};
    }
    ProfileScope ps(MLPMOE_KERNEL_GATE_UP_MFMA, a.stream);
    gate_up_mfma<BMT, WM, NB, S::D, S::kStaged, kRouted><<<(unsigned)grid, WM * 128, 0, a.stream>>>(
        static_cast<const uint16_t *>(a.x), static_cast<const uint16_t *>(a.Wg),
        static_cast<const uint16_t *>(a.Wu), static_cast<uint16_t *>(a.H), a.T, a.d_model, a.d_inter,
        a.ldh, tiles_m, (int)tiles_n, a.route, rt, bt);
    return launch_status("gate_up_mfma launch");
}

static hipError_t launch_gate_up_mixed(const FwdArgs &a, const BranchTable &bt)
{
    const int tiles_m = ceil_div(a.T, BM);
    long long tiles_n = 0;
    for (int r = 0; r < bt.n_runs; ++r) tiles_n += ceil_div(bt.run_end[r] - bt.run_start[r], BNH_MAX);
    const int wide_per_xcd = mixed_wide_per_xcd(tiles_m * tiles_n);
    if (wide_per_xcd < 0) return note_hip_error("gate_up_mfma_mixed: tile count", hipErrorInvalidValue);
    const int rest_per_xcd = ids_per_xcd(tiles_m * tiles_n) - wide_per_xcd;
    const int parts = mixed_rest_parts(tiles_m * tiles_n);
    const long long grid = (long long)XCDS * (wide_per_xcd + (long long)parts * rest_per_xcd);
    ProfileScope ps(MLPMOE_KERNEL_GATE_UP_MFMA, a.stream);
    const auto kernel = parts == 4 ? gate_up_mfma_mixed<MFMA_WM, 4> : gate_up_mfma_mixed<MFMA_WM, 2>;
    kernel<<<(unsigned)grid, MFMA_WM * 128, 0, a.stream>>>(
        static_cast<const uint16_t *>(a.x), static_cast<const uint16_t *>(a.Wg),
        static_cast<const uint16_t *>(a.Wu), static_cast<uint16_t *>(a.H), a.T, a.d_model, a.ldh, tiles_m,
        (int)tiles_n, wide_per_xcd, bt);
    return launch_status("gate_up_mfma_mixed launch");
}

template <typename S, bool kRouted = false>
static hipError_t launch_down(const FwdArgs &a, const BranchTable &bt, int splits)
{
    constexpr int BMT = S::BMT, WM = S::WM, NB = S::NB;
    const int tiles_m = ceil_div(a.T, BMT);
    const int tiles_n = ceil_div(a.d_model, 64 * NB);
    const int kt_total = k_tiles(bt);
    const long long grid = (long long)XCDS * ids_per_xcd((long long)tiles_m * tiles_n * splits);
    if (grid > 0x7fffffffLL) return note_hip_error("down_mfma grid", hipErrorInvalidValue);
    ProfileScope ps(MLPMOE_KERNEL_DOWN_MFMA, a.stream);
    down_mfma<BMT, WM, NB, S::D, S::kStaged, kRouted><<<(unsigned)grid, WM * 128, 0, a.stream>>>(
        static_cast<const uint16_t *>(a.H), static_cast<const uint16_t *>(a.Wd),
        splits > 1 ? a.partial : a.out, a.T, a.d_model, a.d_inter, a.ldh, tiles_m, tiles_n, splits, kt_total,
        (a.out_bf16 && splits == 1) ? DST_BF16 : DST_F32, a.route_scratch, bt);
    return launch_status("down_mfma launch");
}

// The down projection as planned, then the sum of the partial results if K was split through the workspace.
template <bool kRouted>
static hipError_t down_and_reduce(const FwdArgs &a, const BranchTable &bt, const DownPlan &pl)
{
    hipError_t e;
    if (pl.shape == TILE_WIDE) e = launch_down<ShapeWide, kRouted>(a, bt, pl.splits);
    else if (pl.shape == TILE_NARROW) e = launch_down<ShapeNarrow, kRouted>(a, bt, pl.splits);
    else if (kRouted) e = hipErrorInvalidValue;
    else if (pl.shape == TILE_SMALL) e = launch_down<ShapeSmall>(a, bt, pl.splits);
    else if (pl.shape == TILE_DEEP) e = launch_down<ShapeDeep>(a, bt, pl.splits);
    else e = launch_down<ShapeSlim>(a, bt, pl.splits);
    if (e != hipSuccess) return hipErrorLaunchFailure;
    if (pl.splits > 1) {
        ProfileScope ps(MLPMOE_KERNEL_SPLITK_REDUCE, a.stream);
        const size_t n4 = (size_t)a.T * a.d_model / 4;
        size_t blocks = (n4 + 511) / 512;
        if (blocks > 4096) blocks = 4096;
        reduce_partials<<<(unsigned)blocks, 256, 0, a.stream>>>(a.partial, a.out, n4, pl.splits, a.out_bf16 ? 1 : 0);
    }
    return launch_status("reduce_partials launch");
}

// Per-token routing on the MFMA kernels (wide tiles: how many tiles are live is known only on the
// device).  a.route_scratch is route_scratch_bytes(T, d_inter) bytes, 256-byte aligned.
hipError_t launch_mfma_routed_bf16(const FwdArgs &a, const BranchTable &bt)
{
    hipError_t e = launch_gate_up<ShapeWide, true>(a, bt);
    if (e != hipSuccess) return hipErrorLaunchFailure;
    // 256-token tiles (the routing tables are per 256 tokens); narrow when K is split: half the partial sums
    int splits = down_splits(a.T, a.d_model, bt.d_eff, TILE_WIDE);
    const TileShape sh = splits > 1 ? TILE_NARROW : TILE_WIDE;
    splits = std::min(down_splits(a.T, a.d_model, bt.d_eff, sh), std::max(1, k_tiles(bt)));
    if (splits > 1 && (size_t)splits * a.T * a.d_model * sizeof(float) > a.partial_bytes) splits = 1;
    return down_and_reduce<true>(a, bt, DownPlan{sh, splits});
}

hipError_t launch_mfma_bf16(const FwdArgs &a, const BranchTable &bt)
{
    const DownPlan pl = plan_down(a, bt, false);
    TileShape gu = a.tile_shape >= 0 ? (TileShape)a.tile_shape : pick_gate_up_tile(bt, a.T, a.d_model);
    if (gu == TILE_MIXED && mixed_wide_per_xcd(gate_up_tiles(bt, a.T, TILE_WIDE)) < 0) gu = TILE_WIDE;   // forced where it does not apply
    hipError_t e = gu == TILE_WIDE     ? launch_gate_up<ShapeWide>(a, bt)
                   : gu == TILE_NARROW ? launch_gate_up<ShapeNarrow>(a, bt)
                   : gu == TILE_SMALL  ? launch_gate_up<ShapeSmall>(a, bt)
                   : gu == TILE_DEEP   ? launch_gate_up<ShapeDeep>(a, bt)
                   : gu == TILE_SLIM   ? launch_gate_up<ShapeSlim>(a, bt)
                                       : launch_gate_up_mixed(a, bt);
    if (e != hipSuccess) return hipErrorLaunchFailure;
    return down_and_reduce<false>(a, bt, pl);
}

}  // namespace mlpmoe
