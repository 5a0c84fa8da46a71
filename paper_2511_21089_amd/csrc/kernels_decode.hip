// Decode path (T <= 16): bandwidth-bound weight streaming for gfx950.
//
// Every weight element is read exactly once, straight from HBM into MFMA operand registers
// (no LDS staging: there is no reuse to exploit), with the <=16 tokens riding on the N side of
// v_mfma_f32_16x16x32_bf16.  A workgroup owns one tile of 16 weight rows; its waves take
// interleaved 64-element blocks of K, so the workgroup as a whole reads long contiguous
// pieces of every row, and the waves' partial 16x16 results are summed through LDS in a
// fixed order (deterministic).
//
//   decode_gate_up:  rows = neurons of W_gate and W_up, K = d_model,
//                    epilogue h = bf16(alpha_b * SiLU(g) * u)            (Sec. 3.1 inner bracket)
//   decode_down:     rows = output features of W_down, K = active runs of neurons,
//                    epilogue out[t,m] = sum                            (Sec. 3.1 outer sum)
#include "internal.h"

namespace mlpmoe {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int KB = 64;   // K elements per wave step: two MFMA steps, 32 contiguous bytes per lane

__device__ __forceinline__ u32x4 ld16(const uint16_t *p) { return *reinterpret_cast<const u32x4 *>(p); }
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
// and feeds the low 8 to one MFMA and the high 8 to the next; x is loaded with the same
// mapping, so the permutation of K inside a block cancels out.
template <int NW, bool kGateUp>
__global__ void __launch_bounds__(NW * 64)
decode_kernel(const uint16_t *__restrict__ Xin, int ldx, int T,
              const uint16_t *__restrict__ W0, const uint16_t *__restrict__ W1, int ldw,
              int d_model, uint16_t *__restrict__ Hout, int ldh, float *__restrict__ out,
              BranchTable bt)
{
    __shared__ float red[NW][2][256];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r16 = lane & 15, q = lane >> 4;

    // tile -> first row and number of valid rows
    int row0 = 0, row_end = 0;
    if (kGateUp) {
        int tile = blockIdx.x;
        for (int r = 0; r < bt.n_runs; ++r) {
            const int n = (bt.run_end[r] - bt.run_start[r] + 15) / 16;
            if (tile < n) {
                row0 = bt.run_start[r] + tile * 16;
                row_end = bt.run_end[r];
                break;
            }
            tile -= n;
        }
        if (row_end == 0) return;
    } else {
        row0 = blockIdx.x * 16;
        row_end = d_model;
    }
    int wrow = row0 + r16;
    wrow = wrow < row_end ? wrow : row_end - 1;          // clamped rows are computed but never stored
    const uint16_t *w0 = W0 + (size_t)wrow * ldw + q * 16;
    const uint16_t *w1 = kGateUp ? W1 + (size_t)wrow * ldw + q * 16 : nullptr;
    const bool tok = r16 < T;
    const uint16_t *xp = Xin + (size_t)(tok ? r16 : 0) * ldx + q * 16;

    f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
    const u32x4 z = {0, 0, 0, 0};

    const int n_ranges = kGateUp ? 1 : bt.n_runs;
    int skip = wave;                                     // blocks to skip before this wave's next one
    for (int r = 0; r < n_ranges; ++r) {
        const int kbeg = kGateUp ? 0 : bt.run_start[r];
        const int kend = kGateUp ? d_model : bt.run_end[r];
        const int nblk = (kend - kbeg + KB - 1) / KB;
        int blk = skip;
#pragma unroll 4
        for (; blk < nblk; blk += NW) {
            const int k = kbeg + blk * KB;
            const int kl = k + q * 16;
            const bool ok0 = kl < kend, ok1 = kl + 8 < kend;
            const u32x4 a00 = ok0 ? ld16(w0 + k) : z;
            const u32x4 a01 = ok1 ? ld16(w0 + k + 8) : z;
            const u32x4 x0 = (ok0 && tok) ? ld16(xp + k) : z;
            const u32x4 x1 = (ok1 && tok) ? ld16(xp + k + 8) : z;
            acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(a00), as_bf16x8(x0), acc0, 0, 0, 0);
            acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(a01), as_bf16x8(x1), acc0, 0, 0, 0);
            if (kGateUp) {
                const u32x4 a10 = ok0 ? ld16(w1 + k) : z;
                const u32x4 a11 = ok1 ? ld16(w1 + k + 8) : z;
                acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(a10), as_bf16x8(x0), acc1, 0, 0, 0);
                acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(a11), as_bf16x8(x1), acc1, 0, 0, 0);
            }
        }
        skip = blk - nblk;                               // carry the interleave across runs
    }

    // cross-wave sum in wave order
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        red[wave][0][v * 64 + lane] = acc0[v];
        if (kGateUp) red[wave][1][v * 64 + lane] = acc1[v];
    }
    __syncthreads();
    if (threadIdx.x >= 256) return;
    const int v = threadIdx.x >> 6;                      // accumulator register index 0..3
    float s0 = 0.f, s1 = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        s0 += red[w][0][threadIdx.x];
        if (kGateUp) s1 += red[w][1][threadIdx.x];
    }
    // accumulator layout: register v of lane l is D[row 4*(l>>4)+v][col l&15]
    const int row = row0 + 4 * q + v;
    const int t = r16;
    if (t >= T || row >= row_end) return;
    if (kGateUp) {
        const float al = bt.alpha[branch_of(bt, row)];
        Hout[(size_t)t * ldh + row] = to_bf16(al * silu_mul(s0, s1));
    } else {
        out[(size_t)t * d_model + row] = s0;
    }
}

}  // namespace

hipError_t launch_decode_bf16(const FwdArgs &a, const BranchTable &bt)
{
    long long tiles1 = 0;
    for (int r = 0; r < bt.n_runs; ++r) tiles1 += ceil_div(bt.run_end[r] - bt.run_start[r], 16);
    const int tiles2 = ceil_div(a.d_model, 16);
    if (tiles1 > 0x7fffffffLL) return hipErrorInvalidValue;
    const uint16_t *X = static_cast<const uint16_t *>(a.x);
    uint16_t *H = static_cast<uint16_t *>(a.H);
    {
    ProfileScope ps(MLPMOE_KERNEL_DECODE_GATE_UP, a.stream);
    decode_kernel<4, true><<<(unsigned)tiles1, 256, 0, a.stream>>>(
        X, a.d_model, a.T, static_cast<const uint16_t *>(a.Wg), static_cast<const uint16_t *>(a.Wu),
        a.d_model, a.d_model, H, a.ldh, nullptr, bt);
    }
    ProfileScope ps(MLPMOE_KERNEL_DECODE_DOWN, a.stream);
    if (tiles2 >= 192)
        decode_kernel<8, false><<<tiles2, 512, 0, a.stream>>>(
            H, a.ldh, a.T, static_cast<const uint16_t *>(a.Wd), nullptr, a.d_inter, a.d_model, nullptr,
            a.ldh, a.out, bt);
    else
        decode_kernel<16, false><<<tiles2, 1024, 0, a.stream>>>(
            H, a.ldh, a.T, static_cast<const uint16_t *>(a.Wd), nullptr, a.d_inter, a.d_model, nullptr,
            a.ldh, a.out, bt);
    return hipGetLastError();
}

}  // namespace mlpmoe
