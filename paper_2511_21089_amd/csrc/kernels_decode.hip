// Decode path (T <= 16): bandwidth-bound weight streaming for gfx950.
//
// Every weight element is read exactly once, straight from HBM into MFMA operand registers
// (no LDS staging: there is no reuse to exploit), with the <=16 tokens riding on the N side of
// v_mfma_f32_16x16x32_bf16.  A workgroup owns one tile of 16 weight rows; its waves take
// interleaved 64-element blocks of K, so the workgroup as a whole reads long contiguous
// pieces of every row, and the waves' partial 16x16 results are summed through LDS in a
// fixed order (deterministic).
//
//   decode_gate_up:  a tile is 8 neurons: MFMA rows 0-7 are their W_gate rows, rows 8-15 their
//                    W_up rows, K = d_model; epilogue h = bf16(alpha_b * SiLU(g) * u)
//                                                                        (Sec. 3.1 inner bracket)
//   decode_down:     a tile is 16 output features of W_down, K = active runs of neurons,
//                    epilogue out[t,m] = sum                            (Sec. 3.1 outer sum)
//
// Eight-neuron tiles keep the tile count a multiple of the CU count for the usual widths
// (14336 / 8 = 7 * 256) and never straddle a run boundary (boundaries are multiples of 8).
#include <mutex>

#include "internal.h"

namespace mlpmoe {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int KB = 64;   // K elements per wave step: two MFMA steps of 32
// Which 8 of a block's 64 K elements a lane feeds to the two MFMA steps: group q = lane >> 4 takes elements
// q * KQ .. + 7 for the first step and q * KQ + KH .. + 7 for the second.  Any assignment works as long as x
// is loaded the same way (the dot product does not care about the order of K).
constexpr int KQ = 16, KH = 8;

// 16 zero bytes: lanes with nothing to load (token >= T, K chunk past the end of a range) read here.
__device__ const uint32_t g_zero16[4] = {0, 0, 0, 0};

// 16-byte load through the global (not flat) path: every pointer handed in is device memory.
__device__ __forceinline__ u32x4 ld16(const uint16_t *p)
{
    typedef const __attribute__((address_space(1))) u32x4 *gptr;
    return *(gptr)(const void *)p;
}
__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

__device__ __forceinline__ float silu_mul(float g, float u)
{
    const float e = __builtin_amdgcn_exp2f(g * -1.4426950408889634f);
    return g * __builtin_amdgcn_rcpf(1.0f + e) * u;
}

__device__ __forceinline__ uint16_t to_bf16(float v)
{
    const __bf16 b = (__bf16)v;
    return __builtin_bit_cast(uint16_t, b);
}

__device__ __forceinline__ int branch_of(const BranchTable &bt, int j)
{
    int b = 0;
    while (b + 1 < bt.B && j >= bt.off[b + 1]) ++b;
    return b;
}

// Lane layout of v_mfma_f32_16x16x32_bf16: operand lane l holds row/col (l & 15) and the 8
// K values of group q = l >> 4.  A lane here loads 16 contiguous K values k0+16q .. k0+16q+15
// and feeds the low 8 to one MFMA and the high 8 to the next (KQ, KH); x is loaded with the same
// mapping, so the permutation of K inside a block cancels out.  (Giving each MFMA step 64
// contiguous bytes of a row instead was measured and makes no difference.)
//
// Memory-level parallelism: every wave keeps the loads of U of its K blocks in flight (a ring of
// U register sets: block i is consumed, then the load of block i+U is issued into its place).
// All loads are branch free: a lane with nothing to load points at a zero chunk instead.
// Per-token routing (T <= 16): the set of branches some token of the batch takes, as a 64-bit
// word, folded with the active mask.  Every wave works it out for itself from route[T, B]: lane b
// looks down column b.
__device__ __forceinline__ unsigned long long live_branches(const BranchTable &bt, const uint8_t *route, int T)
{
    const int b = threadIdx.x & 63;
    bool any = false;
    if (b < bt.B)
        for (int t = 0; t < T; ++t) any = any || route[(size_t)t * bt.B + b] != 0;
    return __ballot(any) & bt.active;
}

// The stretches of the intermediate dimension a launch works on.  Without routing they are the
// table's runs of active branches; with routing, one stretch per branch, empty unless the branch is
// live (all branch offsets are then multiples of 8).
template <bool kRouted>
struct Stretches {
    const BranchTable &bt;
    unsigned long long live;
    __device__ __forceinline__ int count() const { return kRouted ? bt.B : bt.n_runs; }
    __device__ __forceinline__ int beg(int r) const { return kRouted ? bt.off[r] : bt.run_start[r]; }
    __device__ __forceinline__ int end(int r) const
    {
        if (!kRouted) return bt.run_end[r];
        return ((live >> r) & 1ULL) ? bt.off[r + 1] : bt.off[r];
    }
};

// Walks the groups of 8 rows ("tiles") of the stretches in steps: (stretch, tile inside it).
template <bool kRouted>
struct TileCursor {
    int r, t;
    __device__ __forceinline__ TileCursor(const Stretches<kRouted> &st, int tile) : r(0), t(tile) { settle(st); }
    __device__ __forceinline__ void settle(const Stretches<kRouted> &st)
    {
        while (r < st.count()) {
            const int n = (st.end(r) - st.beg(r)) / 8;   // stretch lengths are multiples of 8
            if (t < n) break;
            t -= n;
            ++r;
        }
    }
    __device__ __forceinline__ void advance(const Stretches<kRouted> &st, int step)
    {
        t += step;
        settle(st);
    }
    // first row of the tile under the cursor, -1 past the last tile
    __device__ __forceinline__ int row0(const Stretches<kRouted> &st) const { return r < st.count() ? st.beg(r) + t * 8 : -1; }
};

template <int NW, int U, bool kGateUp, bool kRouted = false>
__global__ void __launch_bounds__(NW * 64)
decode_kernel(const uint16_t *__restrict__ Xin, int ldx, int T,
              const uint16_t *__restrict__ W0, const uint16_t *__restrict__ W1, int ldw,
              int d_model, uint16_t *__restrict__ Hout, int ldh, float *__restrict__ out, int out_bf16,
              const uint8_t *__restrict__ route, BranchTable bt)
{
    static_assert(NW >= 4, "the final reduction uses 256 threads");
    __shared__ float red[NW][256];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r16 = lane & 15, q = lane >> 4;
    const Stretches<kRouted> st{bt, kRouted ? live_branches(bt, route, T) : 0ULL};

    // tile -> this lane's weight row
    int row0 = 0;
    const uint16_t *wrow;
    if (kGateUp) {
        row0 = TileCursor<kRouted>(st, blockIdx.x).row0(st);
        if (row0 < 0) return;                            // with routing the grid covers all active rows
        wrow = (r16 < 8 ? W0 : W1) + (size_t)(row0 + (r16 & 7)) * ldw;
    } else {
        row0 = blockIdx.x * 16;
        int m = row0 + r16;
        m = m < d_model ? m : d_model - 1;               // clamped rows are computed but never stored
        wrow = W0 + (size_t)m * ldw;
    }
    wrow += q * KQ;
    const bool tok = r16 < T;
    const uint16_t *xp = Xin + (size_t)(tok ? r16 : 0) * ldx + q * KQ;
    const uint16_t *zero = reinterpret_cast<const uint16_t *>(g_zero16);

    // cursor over this wave's blocks: (range, block inside the range); ranges laid end to end
    const int n_ranges = kGateUp ? 1 : st.count();
    auto rbeg = [&](int r) { return kGateUp ? 0 : st.beg(r); };
    auto rend = [&](int r) { return kGateUp ? d_model : st.end(r); };
    int cr = 0, cb = wave;                               // load cursor
    auto settle = [&]() {                                // move past ranges the block index overshoots
        while (cr < n_ranges) {
            const int nb = (rend(cr) - rbeg(cr) + KB - 1) / KB;
            if (cb < nb) break;
            cb -= nb;
            ++cr;
        }
    };
    settle();
    int total = 0;                                       // blocks of this wave in all ranges
    {
        int sk = wave;
        for (int r = 0; r < n_ranges; ++r) {
            const int nb = (rend(r) - rbeg(r) + KB - 1) / KB;
            const int mine = nb > sk ? (nb - sk + NW - 1) / NW : 0;
            total += mine;
            sk = sk + mine * NW - nb;
        }
    }

    u32x4 wa[U][2], xa[U][2];
    auto load_block = [&](int u) {                       // loads the block under the cursor, then advances
        const bool live = cr < n_ranges;
        const int k = live ? rbeg(cr) + cb * KB : 0;
        const int kend = live ? rend(cr) : -1;
        const int kl = k + q * KQ;
        const bool ok0 = kl < kend, ok1 = kl + KH < kend;
        wa[u][0] = ld16(ok0 ? wrow + k : zero);
        wa[u][1] = ld16(ok1 ? wrow + k + KH : zero);
        xa[u][0] = ld16((ok0 && tok) ? xp + k : zero);
        xa[u][1] = ld16((ok1 && tok) ? xp + k + KH : zero);
        cb += NW;
        settle();
    };

    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int u = 0; u < U; ++u) load_block(u);
    for (int j = 0; j < total; j += U) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(wa[u][0]), as_bf16x8(xa[u][0]), acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(wa[u][1]), as_bf16x8(xa[u][1]), acc, 0, 0, 0);
            load_block(u);                               // past the last block this loads zeros
        }
    }

    // cross-wave sum in wave order
#pragma unroll
    for (int v = 0; v < 4; ++v) red[wave][v * 64 + lane] = acc[v];
    __syncthreads();
    if (threadIdx.x >= 256) return;
    // accumulator layout: register v of lane l is D[row 4*(l>>4)+v][col l&15]
    const int v = threadIdx.x >> 6;
    const int row = 4 * q + v;
    const int t = r16;
    if (t >= T) return;
    if (kGateUp) {
        if (row >= 8) return;                            // rows 8-15 hold the up projection of rows 0-7
        float g = 0.f, up = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            g += red[w][threadIdx.x];
            up += red[w][threadIdx.x + 32];              // row + 8: two lane groups further
        }
        const int n = row0 + row;
        const int b = branch_of(bt, n);
        float v = bt.alpha[b] * silu_mul(g, up);
        if (kRouted) v = route[(size_t)t * bt.B + b] ? v : 0.f;
        Hout[(size_t)t * ldh + n] = to_bf16(v);
    } else {
        float s0 = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) s0 += red[w][threadIdx.x];
        const int m = row0 + row;
        if (m < d_model) {
            if (out_bf16)
                reinterpret_cast<uint16_t *>(out)[(size_t)t * d_model + m] = to_bf16(s0);
            else
                out[(size_t)t * d_model + m] = s0;
        }
    }
}

// Down projection with RT row tiles (16 RT output features) per workgroup and the K blocks dealt to TWO
// workgroups (blockIdx.y).  Layers with many output features take RT = 2:  Every workgroup of the one-tile
// kernel reads all of H, which at 16 tokens is as many bytes as its weight rows, all from the same
// L2; here a block of H is used for two weight fragments and each workgroup reads half of H, a quarter
// of that traffic per weight byte, with all CUs still busy.  The two partial sums of an output are
// added into `out` with float atomics: out must hold zeros when the kernel starts (the gate+up
// kernel that runs before it clears it), and 0 + a + b is the same number in either order, so the
// result does not depend on which workgroup comes first.
// Narrow layers (few output features) take RT = 1 with 16 waves: twice the workgroups of the one-tile kernel,
// and a wave's share of K short enough for its ring to hold all of it, so every weight byte is requested
// as the kernel starts.
template <int NW, int U, int RT, bool kRouted = false>
__global__ void __launch_bounds__(NW * 64)
decode_down_split(const uint16_t *__restrict__ Hin, int ldx, int T, const uint16_t *__restrict__ Wd, int ldw,
                  int d_model, float *__restrict__ out, const uint8_t *__restrict__ route, BranchTable bt)
{
    static_assert(NW >= 4, "the final reduction uses 256 threads");
    constexpr int KS = 2;
    __shared__ float red[NW][RT][256];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r16 = lane & 15, q = lane >> 4;
    const Stretches<kRouted> st{bt, kRouted ? live_branches(bt, route, T) : 0ULL};
    const int row0 = blockIdx.x * (16 * RT);
    const uint16_t *wrow[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        int m = row0 + rt * 16 + r16;
        m = m < d_model ? m : d_model - 1;               // clamped rows are computed but never stored
        wrow[rt] = Wd + (size_t)m * ldw + q * KQ;
    }
    const bool tok = r16 < T;
    const uint16_t *xp = Hin + (size_t)(tok ? r16 : 0) * ldx + q * KQ;
    const uint16_t *zero = reinterpret_cast<const uint16_t *>(g_zero16);

    // cursor over this wave's blocks.  The K blocks of all ranges, laid end to end, are cut into KS
    // contiguous parts, one per workgroup (a workgroup then reads long contiguous pieces of its rows);
    // inside its part the waves take the blocks in turn.
    const int n_ranges = st.count();
    int nb_all = 0;
    for (int r = 0; r < n_ranges; ++r) nb_all += (st.end(r) - st.beg(r) + KB - 1) / KB;
    const int part = (nb_all + KS - 1) / KS;
    const int first = wave + (int)blockIdx.y * part, stride = NW;
    const int my_end = (int)(blockIdx.y + 1) * part < nb_all ? (int)(blockIdx.y + 1) * part : nb_all;
    int cr = 0, cb = first;
    auto settle = [&]() {                                // move past ranges the block index overshoots
        while (cr < n_ranges) {
            const int nb = (st.end(cr) - st.beg(cr) + KB - 1) / KB;
            if (cb < nb) break;
            cb -= nb;
            ++cr;
        }
    };
    settle();
    const int total = my_end > first ? (my_end - first + stride - 1) / stride : 0;   // blocks of this wave
    int issued = 0;

    u32x4 wa[U][RT][2], xa[U][2];
    auto load_block = [&](int u) {                       // loads the block under the cursor, then advances
        const bool live = cr < n_ranges && issued < total;     // past its part a wave loads zeros
        ++issued;
        const int k = live ? st.beg(cr) + cb * KB : 0;
        const int kend = live ? st.end(cr) : -1;
        const int kl = k + q * KQ;
        const bool ok0 = kl < kend, ok1 = kl + KH < kend;
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            wa[u][rt][0] = ld16(ok0 ? wrow[rt] + k : zero);
            wa[u][rt][1] = ld16(ok1 ? wrow[rt] + k + KH : zero);
        }
        xa[u][0] = ld16((ok0 && tok) ? xp + k : zero);
        xa[u][1] = ld16((ok1 && tok) ? xp + k + KH : zero);
        cb += stride;
        settle();
    };

    f32x4 acc[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) acc[rt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int u = 0; u < U; ++u) load_block(u);
    for (int j = 0; j < total; j += U) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int rt = 0; rt < RT; ++rt) {
                acc[rt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(wa[u][rt][0]), as_bf16x8(xa[u][0]), acc[rt], 0, 0, 0);
                acc[rt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(wa[u][rt][1]), as_bf16x8(xa[u][1]), acc[rt], 0, 0, 0);
            }
            load_block(u);                               // past the last block this loads zeros
        }
    }

    // cross-wave sum in wave order, then this workgroup's half of K goes into out
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int v = 0; v < 4; ++v) red[wave][rt][v * 64 + lane] = acc[rt][v];
    __syncthreads();
    if (threadIdx.x >= 256) return;
    const int v = threadIdx.x >> 6;
    const int row = 4 * q + v;                           // register v of lane l is D[row 4*(l>>4)+v][col l&15]
    const int t = r16;
    if (t >= T) return;
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        float s0 = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) s0 += red[w][rt][threadIdx.x];
        const int m = row0 + rt * 16 + row;
        if (m < d_model) atomicAdd(&out[(size_t)t * d_model + m], s0);
    }
}

// Persistent gate+up kernel for layers whose x fits in LDS (T * (d_model*2 + 16) bytes).
// One workgroup per CU copies x into LDS once and then walks its tiles (tile t belongs to
// workgroup t % grid, so every CU gets the same number).  The NW waves of the workgroup share each
// tile with interleaved 64-element K blocks, which makes the workgroup read NW*128 contiguous
// bytes of every weight row per step; every wave keeps a ring of U blocks in flight, and the ring
// keeps rolling across tile boundaries, so the loads of the next tile are already under way
// while the partial sums of the current one are reduced through LDS (one barrier per tile, the
// reduction buffer is double buffered).  Each wave's block count per tile is padded to a
// multiple of U with blocks that read a zero chunk, which keeps ring slots compile-time constants.
// x rows are padded by 16 bytes so that the 16 token rows of a fragment fall on distinct banks.
template <int NW, int U, bool kRouted = false>
__global__ void __launch_bounds__(NW * 64)
decode_gate_up_persist(const uint16_t *__restrict__ X, int T, const uint16_t *__restrict__ Wg,
                       const uint16_t *__restrict__ Wu, int d_model, uint16_t *__restrict__ Hout, int ldh,
                       const uint8_t *__restrict__ route, float *__restrict__ clear, int clear_n, BranchTable bt)
{
    // clear (may be null): clear_n floats to set to 0 for the kernel that follows (decode_down_split)
    if (clear)
        for (int i = blockIdx.x * (NW * 64) + threadIdx.x; i < clear_n; i += gridDim.x * (NW * 64)) clear[i] = 0.f;
    static_assert(NW >= 4, "the reduction uses 256 threads");
    extern __shared__ __attribute__((aligned(16))) char smem[];
    float *red = reinterpret_cast<float *>(smem);                 // [2][NW][256]
    char *xs = smem + 2 * NW * 256 * sizeof(float);
    const int row_bytes = d_model * 2 + 16;
    const int zero_off = T * row_bytes;                  // 16 zero bytes after the last row
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r16 = lane & 15, q = lane >> 4;
    const bool tok = r16 < T;
    const int x_lane = (tok ? r16 : 0) * row_bytes + q * (KQ * 2);
    const uint16_t *zero = reinterpret_cast<const uint16_t *>(g_zero16);
    const int nblk = (d_model + KB - 1) / KB;
    const int nb_pad = ((nblk + NW - 1) / NW + U - 1) / U * U;    // blocks per wave per tile, padded
    const size_t lane_row_off = (size_t)(r16 & 7) * d_model + q * KQ;
    const uint16_t *wsel = r16 < 8 ? Wg : Wu;

    // with routing the workgroups share out the tiles of the live branches only
    const Stretches<kRouted> st{bt, kRouted ? live_branches(bt, route, T) : 0ULL};

    // load cursor: U blocks ahead of the block being consumed
    TileCursor<kRouted> l_cur(st, blockIdx.x);
    int l_j = 0;
    int l_row0 = l_cur.row0(st);
    const uint16_t *l_wrow = wsel + (size_t)(l_row0 < 0 ? 0 : l_row0) * d_model + lane_row_off;
    u32x4 wa[U][2];
    auto load_next = [&](int u) {
        const int b = wave + NW * l_j;                   // K block inside the tile
        const int kl = b * KB + q * KQ;
        const bool more = l_row0 >= 0;
        wa[u][0] = ld16((more && kl < d_model) ? l_wrow + b * KB : zero);
        wa[u][1] = ld16((more && kl + KH < d_model) ? l_wrow + b * KB + KH : zero);
        if (++l_j == nb_pad) {
            l_j = 0;
            l_cur.advance(st, gridDim.x);
            l_row0 = l_cur.row0(st);
            if (l_row0 >= 0) l_wrow = wsel + (size_t)l_row0 * d_model + lane_row_off;
        }
    };
#pragma unroll
    for (int u = 0; u < U; ++u) load_next(u);            // the weight stream starts before x is staged

    // x -> LDS, while the first weight blocks are on their way
    {
        const int chunks = T * (d_model / 8);            // 16-byte chunks of x
        for (int i0 = 0; i0 < chunks; i0 += NW * 64 * 8) {
            u32x4 v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {                // 8 loads in flight per thread
                const int i = i0 + j * (NW * 64) + threadIdx.x;
                v[j] = ld16(i < chunks ? X + (size_t)i * 8 : reinterpret_cast<const uint16_t *>(g_zero16));
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int i = i0 + j * (NW * 64) + threadIdx.x;
                if (i < chunks) {
                    const int t = i / (d_model / 8), c = i % (d_model / 8);
                    *reinterpret_cast<u32x4 *>(xs + t * row_bytes + c * 16) = v[j];
                }
            }
        }
    }
    if (threadIdx.x == 0) *reinterpret_cast<u32x4 *>(xs + zero_off) = u32x4{0, 0, 0, 0};
    __syncthreads();

    int it = 0;
    TileCursor<kRouted> cur(st, blockIdx.x);
    for (int row0 = cur.row0(st); row0 >= 0; cur.advance(st, gridDim.x), row0 = cur.row0(st), ++it) {
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
        for (int j0 = 0; j0 < nb_pad; j0 += U) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int b = wave + NW * (j0 + u);
                const int kl = b * KB + q * KQ;
                const int xo0 = (tok && kl < d_model) ? x_lane + b * (KB * 2) : zero_off;
                const int xo1 = (tok && kl + KH < d_model) ? x_lane + b * (KB * 2) + KH * 2 : zero_off;
                const bf16x8 x0 = *reinterpret_cast<const bf16x8 *>(xs + xo0);
                const bf16x8 x1 = *reinterpret_cast<const bf16x8 *>(xs + xo1);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(wa[u][0]), x0, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(wa[u][1]), x1, acc, 0, 0, 0);
                load_next(u);                            // refill the slot just consumed
                __builtin_amdgcn_sched_barrier(0);       // keep the ring rolling: no batching of loads
            }
        }
        // cross-wave sum in wave order; rows 0-7 hold g, rows 8-15 hold u of the same neurons
        float *rb = red + (it & 1) * (NW * 256);
#pragma unroll
        for (int v = 0; v < 4; ++v) rb[wave * 256 + v * 64 + lane] = acc[v];
        __syncthreads();
        if (threadIdx.x < 256) {
            const int v = threadIdx.x >> 6;
            const int row = 4 * q + v;                   // register v of lane l is D[row 4*(l>>4)+v][col l&15]
            if (row < 8 && tok) {
                float g = 0.f, up = 0.f;
#pragma unroll
                for (int w = 0; w < NW; ++w) {
                    g += rb[w * 256 + threadIdx.x];
                    up += rb[w * 256 + threadIdx.x + 32];
                }
                const int n = row0 + row;
                const int b = branch_of(bt, n);
                float v = bt.alpha[b] * silu_mul(g, up);
                if (kRouted) v = route[(size_t)r16 * bt.B + b] ? v : 0.f;
                Hout[(size_t)r16 * ldh + n] = to_bf16(v);
            }
        }
    }
}

// waves and ring depth of the instantiations in use: gate+up fallback, down, persistent gate+up
constexpr int DEC_NW1 = 4, DEC_U1 = 8, DEC_NW2 = 8, DEC_U2 = 8, DEC_SNW = 8, DEC_SU = 8;
// The persistent gate+up kernel with the x fragments held in registers instead of LDS: wave w works on
// K blocks w, w + NW, ... of EVERY tile, so the x fragments it needs are the same for every tile and
// are loaded once, XB blocks of 2 x 16 bytes per lane (d_model <= 64 * NW * XB).  Everything else
// (tile order, ring of U weight blocks rolling across tiles, reduction, epilogue, clear) is
// decode_gate_up_persist's.  XB < U (narrow layers): a revolution of the ring spans U / XB tiles, so the
// weight blocks of that many tiles are in flight per wave and no slot is spent on blocks past d_model.
template <int NW, int U, int XB, bool kRouted = false>
__global__ void __launch_bounds__(NW * 64)
decode_gate_up_xreg(const uint16_t *__restrict__ X, int T, const uint16_t *__restrict__ Wg,
                    const uint16_t *__restrict__ Wu, int d_model, uint16_t *__restrict__ Hout, int ldh,
                    const uint8_t *__restrict__ route, float *__restrict__ clear, int clear_n, BranchTable bt)
{
    if (clear)
        for (int i = blockIdx.x * (NW * 64) + threadIdx.x; i < clear_n; i += gridDim.x * (NW * 64)) clear[i] = 0.f;
    static_assert(NW >= 4 && (XB % U == 0 || U % XB == 0), "the reduction uses 256 threads; ring slots are compile-time");
    constexpr int TPR = XB >= U ? 1 : U / XB;     // tiles per revolution of the ring
    __shared__ float red[2][NW][256];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r16 = lane & 15, q = lane >> 4;
    const bool tok = r16 < T;
    const uint16_t *zero = reinterpret_cast<const uint16_t *>(g_zero16);
    const size_t lane_row_off = (size_t)(r16 & 7) * d_model + q * KQ;
    const uint16_t *wsel = r16 < 8 ? Wg : Wu;
    const Stretches<kRouted> st{bt, kRouted ? live_branches(bt, route, T) : 0ULL};

    TileCursor<kRouted> l_cur(st, blockIdx.x);
    int l_j = 0;
    int l_row0 = l_cur.row0(st);
    const uint16_t *l_wrow = wsel + (size_t)(l_row0 < 0 ? 0 : l_row0) * d_model + lane_row_off;
    u32x4 wa[U][2];
    auto load_next = [&](int u) {
        const int b = wave + NW * l_j;
        const int kl = b * KB + q * KQ;
        const bool more = l_row0 >= 0;
        wa[u][0] = ld16((more && kl < d_model) ? l_wrow + b * KB : zero);
        wa[u][1] = ld16((more && kl + KH < d_model) ? l_wrow + b * KB + KH : zero);
        if (++l_j == XB) {
            l_j = 0;
            l_cur.advance(st, gridDim.x);
            l_row0 = l_cur.row0(st);
            if (l_row0 >= 0) l_wrow = wsel + (size_t)l_row0 * d_model + lane_row_off;
        }
    };
#pragma unroll
    for (int u = 0; u < U; ++u) load_next(u);

    // this wave's x fragments, once
    u32x4 xr[XB][2];
    {
        const uint16_t *xp = X + (size_t)(tok ? r16 : 0) * d_model + q * KQ;
#pragma unroll
        for (int j = 0; j < XB; ++j) {
            const int b = wave + NW * j;
            const int kl = b * KB + q * KQ;
            xr[j][0] = ld16((tok && kl < d_model) ? xp + b * KB : zero);
            xr[j][1] = ld16((tok && kl + KH < d_model) ? xp + b * KB + KH : zero);
        }
    }

    int it = 0;
    TileCursor<kRouted> cur(st, blockIdx.x);
    int row0 = cur.row0(st);
    while (row0 >= 0) {
#pragma unroll
        for (int tt = 0; tt < TPR; ++tt) {           // tile tt of this revolution uses ring slots tt * XB ...
            if (row0 < 0) break;
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int j0 = 0; j0 < XB; j0 += U) {
#pragma unroll
                for (int ju = 0; ju < (XB < U ? XB : U); ++ju) {
                    const int u = XB < U ? tt * XB + ju : ju;
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(wa[u][0]), as_bf16x8(xr[j0 + ju][0]), acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(wa[u][1]), as_bf16x8(xr[j0 + ju][1]), acc, 0, 0, 0);
                    load_next(u);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            float *rb = &red[it & 1][0][0];
#pragma unroll
            for (int v = 0; v < 4; ++v) rb[wave * 256 + v * 64 + lane] = acc[v];
            __syncthreads();
            if (threadIdx.x < 256) {
                const int v = threadIdx.x >> 6;
                const int row = 4 * q + v;
                if (row < 8 && tok) {
                    float g = 0.f, up = 0.f;
#pragma unroll
                    for (int w = 0; w < NW; ++w) {
                        g += rb[w * 256 + threadIdx.x];
                        up += rb[w * 256 + threadIdx.x + 32];
                    }
                    const int n = row0 + row;
                    const int b = branch_of(bt, n);
                    float v = bt.alpha[b] * silu_mul(g, up);
                    if (kRouted) v = route[(size_t)r16 * bt.B + b] ? v : 0.f;
                    Hout[(size_t)r16 * ldh + n] = to_bf16(v);
                }
            }
            ++it;
            cur.advance(st, gridDim.x);
            row0 = cur.row0(st);
        }
    }
}

constexpr size_t kStreamLdsMax = 160 * 1024;

}  // namespace

template <bool kRouted>
static hipError_t launch_decode_impl(const FwdArgs &a, const BranchTable &bt)
{
    long long tiles1 = 0;
    for (int r = 0; r < bt.n_runs; ++r) tiles1 += (bt.run_end[r] - bt.run_start[r]) / 8;
    const int tiles2 = ceil_div(a.d_model, 16);
    if (tiles1 > 0x7fffffffLL) return hipErrorInvalidValue;
    const uint16_t *X = static_cast<const uint16_t *>(a.x);
    uint16_t *H = static_cast<uint16_t *>(a.H);
    const size_t xs_bytes = (size_t)a.T * (a.d_model * 2 + 16) + 16 + 2 * DEC_SNW * 256 * sizeof(float);
    // blocks of K per wave and tile in the persistent kernels, padded to whole ring revolutions
    const int nb_pad = ceil_div(ceil_div(ceil_div(a.d_model, KB), DEC_SNW), DEC_SU) * DEC_SU;
    const bool x_in_regs = nb_pad <= 16;                    // d_model <= 8192: x fragments stay in registers
    const bool persistent = x_in_regs || xs_bytes <= kStreamLdsMax;
    // A float result comes from the down kernel that splits K over two workgroups and adds the halves
    // into `out` with atomics; `out` is cleared by the persistent gate+up kernel, so the pair is only used
    // together.
    const bool split_down = persistent && !a.out_bf16;
    float *clear = split_down ? a.out : nullptr;
    const int clear_n = split_down ? a.T * a.d_model : 0;
    const uint16_t *Wg = static_cast<const uint16_t *>(a.Wg), *Wu = static_cast<const uint16_t *>(a.Wu);
    if (persistent) {
        // per device, set up on the first call there: CU count and the LDS limit of the kernel that stages x
        static std::mutex mu;
        static int cus_of[64] = {0};              // one table per instantiation (attribute is per kernel)
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return note_hip_error("hipGetDevice", e);
        if (dev < 0 || dev >= 64) return note_hip_error("device index", hipErrorInvalidDevice);
        int n_cus;
        {
            std::lock_guard<std::mutex> lock(mu);
            if (cus_of[dev] == 0) {
                hipDeviceProp_t prop;
                e = hipGetDeviceProperties(&prop, dev);
                if (e != hipSuccess) return note_hip_error("hipGetDeviceProperties", e);
                e = hipFuncSetAttribute(
                    reinterpret_cast<const void *>(&decode_gate_up_persist<DEC_SNW, DEC_SU, kRouted>),
                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)kStreamLdsMax);
                if (e != hipSuccess) return note_hip_error("hipFuncSetAttribute(decode_gate_up_persist)", e);
                cus_of[dev] = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 1;
            }
            n_cus = cus_of[dev];
        }
        const int grid = tiles1 < n_cus ? (int)tiles1 : n_cus;
        ProfileScope ps(MLPMOE_KERNEL_DECODE_GATE_UP, a.stream);
        const int nb_wave = ceil_div(ceil_div(a.d_model, KB), DEC_SNW);      // K blocks per wave and tile
        if (nb_wave <= 2)
            decode_gate_up_xreg<DEC_SNW, DEC_SU, 2, kRouted><<<grid, DEC_SNW * 64, 0, a.stream>>>(
                X, a.T, Wg, Wu, a.d_model, H, a.ldh, a.route, clear, clear_n, bt);
        else if (nb_wave <= 4)
            decode_gate_up_xreg<DEC_SNW, DEC_SU, 4, kRouted><<<grid, DEC_SNW * 64, 0, a.stream>>>(
                X, a.T, Wg, Wu, a.d_model, H, a.ldh, a.route, clear, clear_n, bt);
        else if (nb_pad <= 8)
            decode_gate_up_xreg<DEC_SNW, DEC_SU, 8, kRouted><<<grid, DEC_SNW * 64, 0, a.stream>>>(
                X, a.T, Wg, Wu, a.d_model, H, a.ldh, a.route, clear, clear_n, bt);
        else if (nb_pad <= 16)
            decode_gate_up_xreg<DEC_SNW, DEC_SU, 16, kRouted><<<grid, DEC_SNW * 64, 0, a.stream>>>(
                X, a.T, Wg, Wu, a.d_model, H, a.ldh, a.route, clear, clear_n, bt);
        else
            decode_gate_up_persist<DEC_SNW, DEC_SU, kRouted><<<grid, DEC_SNW * 64, xs_bytes, a.stream>>>(
                X, a.T, Wg, Wu, a.d_model, H, a.ldh, a.route, clear, clear_n, bt);
        if (launch_status("decode gate+up (persistent) launch") != hipSuccess) return hipErrorLaunchFailure;
    } else {
        ProfileScope ps(MLPMOE_KERNEL_DECODE_GATE_UP, a.stream);
        decode_kernel<DEC_NW1, DEC_U1, true, kRouted><<<(unsigned)tiles1, DEC_NW1 * 64, 0, a.stream>>>(
            X, a.d_model, a.T, Wg, Wu, a.d_model, a.d_model, H, a.ldh, nullptr, 0, a.route, bt);
        if (launch_status("decode gate_up launch") != hipSuccess) return hipErrorLaunchFailure;
    }
    ProfileScope ps(MLPMOE_KERNEL_DECODE_DOWN, a.stream);
    if (split_down && tiles2 >= 192)
        decode_down_split<4, 8, 2, kRouted><<<dim3(ceil_div(a.d_model, 32), 2), 4 * 64, 0, a.stream>>>(
            H, a.ldh, a.T, static_cast<const uint16_t *>(a.Wd), a.d_inter, a.d_model, a.out, a.route, bt);
    else if (split_down)
        decode_down_split<16, 4, 1, kRouted><<<dim3(tiles2, 2), 16 * 64, 0, a.stream>>>(
            H, a.ldh, a.T, static_cast<const uint16_t *>(a.Wd), a.d_inter, a.d_model, a.out, a.route, bt);
    else if (tiles2 >= 192)
        decode_kernel<DEC_NW2, DEC_U2, false, kRouted><<<tiles2, DEC_NW2 * 64, 0, a.stream>>>(
            H, a.ldh, a.T, static_cast<const uint16_t *>(a.Wd), nullptr, a.d_inter, a.d_model, nullptr,
            a.ldh, a.out, a.out_bf16 ? 1 : 0, a.route, bt);
    else
        decode_kernel<16, 4, false, kRouted><<<tiles2, 1024, 0, a.stream>>>(
            H, a.ldh, a.T, static_cast<const uint16_t *>(a.Wd), nullptr, a.d_inter, a.d_model, nullptr,
            a.ldh, a.out, a.out_bf16 ? 1 : 0, a.route, bt);
    return launch_status("decode_down launch");
}

hipError_t launch_decode_bf16(const FwdArgs &a, const BranchTable &bt) { return launch_decode_impl<false>(a, bt); }

// Per-token routing, T <= 16: the kernels read a.route themselves and need no scratch.
hipError_t launch_decode_routed_bf16(const FwdArgs &a, const BranchTable &bt) { return launch_decode_impl<true>(a, bt); }

}  // namespace mlpmoe
