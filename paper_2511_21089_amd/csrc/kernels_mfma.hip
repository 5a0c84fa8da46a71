// Prefill path: bf16 MFMA kernels for gfx950 (v_mfma_f32_32x32x16_bf16, wave64).
//
// Kernel 1  gate_up_mfma:  H[t,j] = bf16( alpha_b(j) * SiLU(<x_t,Wg_j>) * <x_t,Wu_j> )
//           one 256-token x 128-neuron tile per workgroup with TWO fp32 accumulator sets
//           (gate and up), so the gated product of Sec. 3.1's inner bracket is formed in
//           registers and only H (bf16) leaves the CU.
// Kernel 2  down_mfma:     out[t,m] = sum_{j in active runs} H[t,j] * Wd[m,j]
//           one 256x256 tile per workgroup; the K loop walks every active run back to back,
//           so the sum over branches of Sec. 3.1 is one fp32 accumulation with no per-branch
//           round trip.  Small outputs are split along K into deterministic partial sums.
//
// Both kernels share one main loop: A rows (tokens) against two blocks of 128 B rows,
// 4 waves in a 2x2 arrangement, each wave owning 128 x (64+64) outputs = 16 MFMA tiles.
#include "internal.h"

namespace mlpmoe {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int BM = 256;          // tokens per tile
constexpr int BNH = 128;         // rows of each of the two B blocks
constexpr int BK = 64;           // K elements per stage
constexpr int THREADS = 256;
constexpr int LDS_ROW = BK + 8;  // padded row (elements): 144 B keeps ds_read_b128 conflict free
constexpr int STAGE_ELEMS = (BM + 2 * BNH) * LDS_ROW;
constexpr int A_CHUNKS = BM * (BK / 8) / THREADS;    // 16-byte chunks per thread: 8
constexpr int B_CHUNKS = BNH * (BK / 8) / THREADS;   // 4 per block

struct TileRegs {
    u32x4 a[A_CHUNKS], b0[B_CHUNKS], b1[B_CHUNKS];
};

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
    c.run = kr.n_runs();
    return c;
}

__device__ __forceinline__ u32x4 ld16(const uint16_t *p) { return *reinterpret_cast<const u32x4 *>(p); }

// Main loop.  A: [*, lda] rows a_row0.. (clamped to a_rows-1), B0/B1: [*, ldb] rows.
// K tiles [kt_begin, kt_end) of the flattened range list kr.
// Rows outside the valid range are clamped to a valid row: their results are never stored,
// and MFMA rows/columns do not mix.  K chunks outside a run are zero in A and in B.
template <typename KR>
__device__ __forceinline__ void mainloop(const uint16_t *__restrict__ A, int lda, int a_row0, int a_rows,
                                         const uint16_t *__restrict__ B0, const uint16_t *__restrict__ B1,
                                         int ldb, int b0_row0, int b1_row0, int b_rows,
                                         const KR &kr, int kt_begin, int kt_end,
                                         uint16_t *lds, f32x16 (&acc0)[4][2], f32x16 (&acc1)[4][2])
{
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int kc = tid & 7;                  // 16-byte chunk inside the 128-byte tile row
    const int r_in = tid >> 3;               // 0..31: row inside a 32-row slab

    const uint16_t *a_ptr[A_CHUNKS];
    const uint16_t *b0_ptr[B_CHUNKS], *b1_ptr[B_CHUNKS];
#pragma unroll
    for (int i = 0; i < A_CHUNKS; ++i) {
        int r = a_row0 + i * 32 + r_in;
        r = r < a_rows ? r : a_rows - 1;
        a_ptr[i] = A + (size_t)r * lda + kc * 8;
    }
#pragma unroll
    for (int i = 0; i < B_CHUNKS; ++i) {
        int r0 = b0_row0 + i * 32 + r_in, r1 = b1_row0 + i * 32 + r_in;
        r0 = r0 < b_rows ? r0 : b_rows - 1;
        r1 = r1 < b_rows ? r1 : b_rows - 1;
        b0_ptr[i] = B0 + (size_t)r0 * ldb + kc * 8;
        b1_ptr[i] = B1 + (size_t)r1 * ldb + kc * 8;
    }

    auto load_tile = [&](const KCursor &c, TileRegs &t) {
        if (c.k + BK <= kr.end(c.run)) {     // whole tile inside the range (uniform branch)
#pragma unroll
            for (int i = 0; i < A_CHUNKS; ++i) t.a[i] = ld16(a_ptr[i] + c.k);
#pragma unroll
            for (int i = 0; i < B_CHUNKS; ++i) {
                t.b0[i] = ld16(b0_ptr[i] + c.k);
                t.b1[i] = ld16(b1_ptr[i] + c.k);
            }
        } else {                             // last tile of a range: chunks past its end are zero
            const bool ok = c.k + kc * 8 < kr.end(c.run);
            const u32x4 z = {0, 0, 0, 0};
#pragma unroll
            for (int i = 0; i < A_CHUNKS; ++i) t.a[i] = ok ? ld16(a_ptr[i] + c.k) : z;
#pragma unroll
            for (int i = 0; i < B_CHUNKS; ++i) {
                t.b0[i] = ok ? ld16(b0_ptr[i] + c.k) : z;
                t.b1[i] = ok ? ld16(b1_ptr[i] + c.k) : z;
            }
        }
    };
    auto store_tile = [&](const TileRegs &t, uint16_t *stage) {
        uint16_t *sa = stage, *sb0 = stage + BM * LDS_ROW, *sb1 = sb0 + BNH * LDS_ROW;
#pragma unroll
        for (int i = 0; i < A_CHUNKS; ++i)
            *reinterpret_cast<u32x4 *>(sa + (i * 32 + r_in) * LDS_ROW + kc * 8) = t.a[i];
#pragma unroll
        for (int i = 0; i < B_CHUNKS; ++i) {
            *reinterpret_cast<u32x4 *>(sb0 + (i * 32 + r_in) * LDS_ROW + kc * 8) = t.b0[i];
            *reinterpret_cast<u32x4 *>(sb1 + (i * 32 + r_in) * LDS_ROW + kc * 8) = t.b1[i];
        }
    };
    auto advance = [&](KCursor &c) {
        c.k += BK;
        if (c.k >= kr.end(c.run)) {
            ++c.run;
            c.k = c.run < kr.n_runs() ? kr.start(c.run) : 0;
        }
    };

    const int nk = kt_end - kt_begin;
    if (nk <= 0) return;
    KCursor cur = k_seek(kr, kt_begin);
    TileRegs regs;
    load_tile(cur, regs);
    store_tile(regs, lds);
    __syncthreads();

    // per-lane read offsets inside a stage (elements)
    const int lrow = lane & 31, lk = (lane >> 5) * 8;
    const int a_off = (wm * 128 + lrow) * LDS_ROW + lk;
    const int b_off = (wn * 64 + lrow) * LDS_ROW + lk;

    for (int it = 0; it < nk; ++it) {
        uint16_t *stage = lds + (it & 1) * STAGE_ELEMS;
        const bool more = it + 1 < nk;
        if (more) {
            advance(cur);
            load_tile(cur, regs);
        }
        const uint16_t *sa = stage + a_off;
        const uint16_t *sb0 = stage + BM * LDS_ROW + b_off;
        const uint16_t *sb1 = sb0 + BNH * LDS_ROW;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8 af[4], bf0[2], bf1[2];
#pragma unroll
            for (int i = 0; i < 4; ++i)
                af[i] = *reinterpret_cast<const bf16x8 *>(sa + i * 32 * LDS_ROW + ks * 16);
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                bf0[j] = *reinterpret_cast<const bf16x8 *>(sb0 + j * 32 * LDS_ROW + ks * 16);
                bf1[j] = *reinterpret_cast<const bf16x8 *>(sb1 + j * 32 * LDS_ROW + ks * 16);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    acc0[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bf0[j], acc0[i][j], 0, 0, 0);
                    acc1[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bf1[j], acc1[i][j], 0, 0, 0);
                }
        }
        if (more) store_tile(regs, lds + ((it + 1) & 1) * STAGE_ELEMS);
        __syncthreads();
    }
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

// grid.x = tilesM * (sum over runs of N tiles); tile id -> (m tile fastest, n tile).
__global__ void __launch_bounds__(THREADS)
gate_up_mfma(const uint16_t *__restrict__ X, const uint16_t *__restrict__ Wg,
             const uint16_t *__restrict__ Wu, uint16_t *__restrict__ H, int T, int d_model, int d_inter,
             int ldh, int tiles_m, BranchTable bt)
{
    __shared__ __attribute__((aligned(16))) uint16_t lds[2 * STAGE_ELEMS];
    const int tm = blockIdx.x % tiles_m;
    int tn = blockIdx.x / tiles_m;
    int n0 = 0, n_end = 0;
    for (int r = 0; r < bt.n_runs; ++r) {
        const int n = (bt.run_end[r] - bt.run_start[r] + BNH - 1) / BNH;
        if (tn < n) {
            n0 = bt.run_start[r] + tn * BNH;
            n_end = bt.run_end[r];
            break;
        }
        tn -= n;
    }
    if (n_end == 0) return;
    const int t0 = tm * BM;

    f32x16 accg[4][2], accu[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                accg[i][j][v] = 0.f;
                accu[i][j][v] = 0.f;
            }

    const int nk = (d_model + BK - 1) / BK;
    mainloop(X, d_model, t0, T, Wg, Wu, d_model, n0, n0, n_end, KSingle{d_model}, 0, nk, lds, accg, accu);

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave >> 1, wn = wave & 1;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int n = n0 + wn * 64 + j * 32 + (lane & 31);
        if (n >= n_end) continue;
        const float al = bt.alpha[branch_of(bt, n)];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int t = t0 + wm * 128 + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                if (t < T) H[(size_t)t * ldh + n] = to_bf16(al * silu_mul(accg[i][j][v], accu[i][j][v]));
            }
        }
    }
}

// grid.x = tilesM * tilesN * splits; dst = out (splits == 1) or partial[split][T][d_model].
__global__ void __launch_bounds__(THREADS)
down_mfma(const uint16_t *__restrict__ H, const uint16_t *__restrict__ Wd, float *__restrict__ dst, int T,
          int d_model, int d_inter, int ldh, int tiles_m, int tiles_n, int splits, int kt_total,
          BranchTable bt)
{
    __shared__ __attribute__((aligned(16))) uint16_t lds[2 * STAGE_ELEMS];
    int id = blockIdx.x;
    const int tm = id % tiles_m;
    id /= tiles_m;
    const int tn = id % tiles_n;
    const int z = id / tiles_n;
    const int t0 = tm * BM, n0 = tn * (2 * BNH);
    const int kt_begin = (int)((long long)kt_total * z / splits);
    const int kt_end = (int)((long long)kt_total * (z + 1) / splits);

    f32x16 acc0[4][2], acc1[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                acc0[i][j][v] = 0.f;
                acc1[i][j][v] = 0.f;
            }

    mainloop(H, ldh, t0, T, Wd, Wd, d_inter, n0, n0 + BNH, d_model, KRuns{bt}, kt_begin, kt_end, lds,
             acc0, acc1);

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    float *o = dst + (size_t)z * T * d_model;
#pragma unroll
    for (int half = 0; half < 2; ++half)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int n = n0 + half * BNH + wn * 64 + j * 32 + (lane & 31);
            if (n >= d_model) continue;
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int t = t0 + wm * 128 + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                    if (t < T) o[(size_t)t * d_model + n] = half ? acc1[i][j][v] : acc0[i][j][v];
                }
        }
}

// out[i] = sum_z partial[z][i], summed in z order: deterministic.
__global__ void reduce_partials(const float *__restrict__ partial, float *__restrict__ out, size_t n,
                                int splits)
{
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n;
         i += (size_t)gridDim.x * blockDim.x) {
        float s = partial[i];
        for (int z = 1; z < splits; ++z) s += partial[(size_t)z * n + i];
        out[i] = s;
    }
}

int k_tiles(const BranchTable &bt)
{
    int n = 0;
    for (int r = 0; r < bt.n_runs; ++r) n += ceil_div(bt.run_end[r] - bt.run_start[r], BK);
    return n;
}

}  // namespace

int mfma_down_splits(int T, int d_model, int k_elems)
{
    const long long tiles = (long long)ceil_div(T, BM) * ceil_div(d_model, 2 * BNH);
    const int kt = ceil_div(k_elems > 0 ? k_elems : 1, BK);
    long long s = 256 / tiles;
    if (s > kt / 4) s = kt / 4;
    if (s > 32) s = 32;
    return s < 1 ? 1 : (int)s;
}

size_t mfma_partial_bytes(int T, int d_model, int d_inter)
{
    const int s = mfma_down_splits(T, d_model, d_inter);
    return s > 1 ? align_up((size_t)s * T * d_model * sizeof(float), 256) : 0;
}

hipError_t launch_mfma_bf16(const FwdArgs &a, const BranchTable &bt)
{
    const int tiles_m = ceil_div(a.T, BM);
    long long tiles_n1 = 0;
    for (int r = 0; r < bt.n_runs; ++r) tiles_n1 += ceil_div(bt.run_end[r] - bt.run_start[r], BNH);
    const long long grid1 = tiles_m * tiles_n1;
    const int tiles_n2 = ceil_div(a.d_model, 2 * BNH);
    // splits from the active width: never more than the workspace was sized for (d_inter >= d_eff)
    int splits = mfma_down_splits(a.T, a.d_model, bt.d_eff);
    const int kt_total = k_tiles(bt);
    if (splits > kt_total) splits = kt_total;
    if (splits > 1 && (size_t)splits * a.T * a.d_model * sizeof(float) > a.partial_bytes) splits = 1;
    const long long grid2 = (long long)tiles_m * tiles_n2 * splits;
    if (grid1 > 0x7fffffffLL || grid2 > 0x7fffffffLL) return hipErrorInvalidValue;

    {
    ProfileScope ps(MLPMOE_KERNEL_GATE_UP_MFMA, a.stream);
    gate_up_mfma<<<(unsigned)grid1, THREADS, 0, a.stream>>>(
        static_cast<const uint16_t *>(a.x), static_cast<const uint16_t *>(a.Wg),
        static_cast<const uint16_t *>(a.Wu), static_cast<uint16_t *>(a.H), a.T, a.d_model, a.d_inter,
        a.ldh, tiles_m, bt);
    }
    float *dst = splits > 1 ? a.partial : a.out;
    {
    ProfileScope ps(MLPMOE_KERNEL_DOWN_MFMA, a.stream);
    down_mfma<<<(unsigned)grid2, THREADS, 0, a.stream>>>(
        static_cast<const uint16_t *>(a.H), static_cast<const uint16_t *>(a.Wd), dst, a.T, a.d_model,
        a.d_inter, a.ldh, tiles_m, tiles_n2, splits, kt_total, bt);
    }
    if (splits > 1) {
        ProfileScope ps(MLPMOE_KERNEL_SPLITK_REDUCE, a.stream);
        const size_t n = (size_t)a.T * a.d_model;
        size_t blocks = (n + 255) / 256;
        if (blocks > 8192) blocks = 8192;
        reduce_partials<<<(unsigned)blocks, 256, 0, a.stream>>>(a.partial, a.out, n, splits);
    }
    return hipGetLastError();
}

}  // namespace mlpmoe
