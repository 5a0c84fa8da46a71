// Generic path: LDS-tiled FMA kernels that accept any shape and alignment.
// Serves the float entry points and bf16 calls whose branch boundaries are not
// multiples of 8 neurons.  Also holds the zero-fill and weight-compaction kernels.
//
// Step 1 (Sec. 3.1, inner bracket):  H[t,j] = alpha_b(j) * SiLU(<x_t, Wg_j>) * <x_t, Wu_j>
// Step 2 (Sec. 3.1, outer product and sum over b):  out[t,m] = sum_{j active} H[t,j] * Wd[m,j]
#include "internal.h"

namespace mlpmoe {
namespace {

constexpr int GT = 64;    // output tile edge
constexpr int GK = 16;    // K step
constexpr int GTHREADS = 256;

__device__ __forceinline__ float load_as_float(const float *p, size_t i) { return p[i]; }
__device__ __forceinline__ float load_as_float(const uint16_t *p, size_t i)
{
    return __uint_as_float((uint32_t)p[i] << 16);
}

__device__ __forceinline__ uint16_t float_to_bf16_rne(float v)
{
    uint32_t u = __float_as_uint(v);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

__device__ __forceinline__ void store_h(float *H, size_t i, float v) { H[i] = v; }
__device__ __forceinline__ void store_h(uint16_t *H, size_t i, float v) { H[i] = float_to_bf16_rne(v); }

// Branch of neuron j, or -1 if j lies in an inactive branch.
__device__ __forceinline__ int branch_of(const BranchTable &bt, int j)
{
    int b = 0;
    while (b + 1 < bt.B && j >= bt.off[b + 1]) ++b;
    return ((bt.active >> b) & 1ULL) ? b : -1;
}

// One thread owns a 4x4 patch of a 64x64 tile; rows come from A (tokens), columns from the B rows.
template <typename TIn, typename TH>
__global__ void __launch_bounds__(GTHREADS)
gate_up_generic(const TIn *__restrict__ X, const TIn *__restrict__ Wg, const TIn *__restrict__ Wu,
                TH *__restrict__ H, int T, int K, int d_inter, int ldh, const uint8_t *__restrict__ route,
                BranchTable bt)
{
    // route (may be null): per-token routing [T, B]; H is 0 where a token does not take a branch
    __shared__ float Xs[GK][GT + 1], Gs[GK][GT + 1], Us[GK][GT + 1];
    const int t0 = blockIdx.y * GT, n0 = blockIdx.x * GT;
    // skip tiles that hold no active neuron
    bool any = false;
    for (int r = 0; r < bt.n_runs; ++r)
        any |= (bt.run_start[r] < n0 + GT) && (bt.run_end[r] > n0);
    if (!any) return;

    const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
    float g[4][4] = {}, u[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += GK) {
        for (int i = threadIdx.x; i < GT * GK; i += GTHREADS) {
            const int r = i / GK, kk = i % GK;
            const bool kin = k0 + kk < K;
            const int t = t0 + r, n = n0 + r;
            Xs[kk][r] = (kin && t < T) ? load_as_float(X, (size_t)t * K + k0 + kk) : 0.f;
            const bool nin = kin && n < d_inter;
            Gs[kk][r] = nin ? load_as_float(Wg, (size_t)n * K + k0 + kk) : 0.f;
            Us[kk][r] = nin ? load_as_float(Wu, (size_t)n * K + k0 + kk) : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < GK; ++kk) {
            float xv[4], gv[4], uv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                xv[i] = Xs[kk][ty * 4 + i];
                gv[i] = Gs[kk][tx * 4 + i];
                uv[i] = Us[kk][tx * 4 + i];
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    g[i][j] = fmaf(xv[i], gv[j], g[i][j]);
                    u[i][j] = fmaf(xv[i], uv[j], u[i][j]);
                }
        }
        __syncthreads();
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int n = n0 + tx * 4 + j;
        if (n >= d_inter) continue;
        const int b = branch_of(bt, n);
        if (b < 0) continue;                 // pruned branch: H is neither written nor read
        const float al = bt.alpha[b];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int t = t0 + ty * 4 + i;
            if (t >= T) continue;
            const float gg = g[i][j];
            const float s = gg / (1.0f + expf(-gg));
            float v = al * (s * u[i][j]);
            if (route && !route[(size_t)t * bt.B + b]) v = 0.f;
            store_h(H, (size_t)t * ldh + n, v);
        }
    }
}

template <typename TIn, typename TH>
__device__ __forceinline__ float h_as_float(const TH *H, size_t i);
template <>
__device__ __forceinline__ float h_as_float<float, float>(const float *H, size_t i) { return H[i]; }
template <>
__device__ __forceinline__ float h_as_float<uint16_t, uint16_t>(const uint16_t *H, size_t i)
{
    return __uint_as_float((uint32_t)H[i] << 16);
}

template <typename TIn, typename TH>
__global__ void __launch_bounds__(GTHREADS)
down_generic(const TH *__restrict__ H, const TIn *__restrict__ Wd, float *__restrict__ out, int out_bf16,
             int T, int d_model, int d_inter, int ldh, BranchTable bt)
{
    __shared__ float Hs[GK][GT + 1], Ds[GK][GT + 1];
    const int t0 = blockIdx.y * GT, m0 = blockIdx.x * GT;
    const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
    float acc[4][4] = {};
    for (int r = 0; r < bt.n_runs; ++r) {
        const int kend = bt.run_end[r];
        for (int k0 = bt.run_start[r]; k0 < kend; k0 += GK) {
            for (int i = threadIdx.x; i < GT * GK; i += GTHREADS) {
                const int rr = i / GK, kk = i % GK;
                const bool kin = k0 + kk < kend;       // never touch columns of a pruned branch
                const int t = t0 + rr, m = m0 + rr;
                Hs[kk][rr] = (kin && t < T) ? h_as_float<TIn, TH>(H, (size_t)t * ldh + k0 + kk) : 0.f;
                Ds[kk][rr] = (kin && m < d_model) ? load_as_float(Wd, (size_t)m * d_inter + k0 + kk) : 0.f;
            }
            __syncthreads();
#pragma unroll
            for (int kk = 0; kk < GK; ++kk) {
                float hv[4], dv[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    hv[i] = Hs[kk][ty * 4 + i];
                    dv[i] = Ds[kk][tx * 4 + i];
                }
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(hv[i], dv[j], acc[i][j]);
            }
            __syncthreads();
        }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int t = t0 + ty * 4 + i;
        if (t >= T) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int m = m0 + tx * 4 + j;
            if (m >= d_model) continue;
            if (out_bf16)
                reinterpret_cast<uint16_t *>(out)[(size_t)t * d_model + m] = float_to_bf16_rne(acc[i][j]);
            else
                out[(size_t)t * d_model + m] = acc[i][j];
        }
    }
}

template <typename Tel>
__global__ void fill_zero_kernel(Tel *out, size_t n)
{
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n;
         i += (size_t)gridDim.x * blockDim.x)
        out[i] = (Tel)0;
}

// Row gather for W_gate / W_up (grid.y = destination row) and column gather for W_down
// (grid.y = row of W_down).  T is a 2- or 4-byte unsigned integer: pure data movement.
template <typename Tel>
__global__ void gather_rows_kernel(const Tel *__restrict__ src, const int32_t *__restrict__ gather,
                                   Tel *__restrict__ dst, int d_model)
{
    const int r = blockIdx.y;
    const int g = gather[r];
    for (int k = blockIdx.x * blockDim.x + threadIdx.x; k < d_model; k += gridDim.x * blockDim.x)
        dst[(size_t)r * d_model + k] = g >= 0 ? src[(size_t)g * d_model + k] : (Tel)0;
}

template <typename Tel>
__global__ void gather_cols_kernel(const Tel *__restrict__ src, const int32_t *__restrict__ gather,
                                   Tel *__restrict__ dst, int n_rows, int d_inter_src)
{
    const int m = blockIdx.y;
    for (int r = blockIdx.x * blockDim.x + threadIdx.x; r < n_rows; r += gridDim.x * blockDim.x) {
        const int g = gather[r];
        dst[(size_t)m * n_rows + r] = g >= 0 ? src[(size_t)m * d_inter_src + g] : (Tel)0;
    }
}

template <typename Tel>
hipError_t compact_typed(const void *Wg, const void *Wu, const void *Wd, const int32_t *gather,
                         int n_rows, int d_model, int d_inter_src, void *Wg_c, void *Wu_c, void *Wd_c,
                         hipStream_t s)
{
    // grid.y is limited to 65535: walk it in slabs
    const int bx = ceil_div(d_model, 256) < 64 ? ceil_div(d_model, 256) : 64;
    for (int r0 = 0; r0 < n_rows; r0 += 32768) {
        const int nr = n_rows - r0 < 32768 ? n_rows - r0 : 32768;
        dim3 grid(bx, nr);
        gather_rows_kernel<Tel><<<grid, 256, 0, s>>>(static_cast<const Tel *>(Wg), gather + r0,
                                                     static_cast<Tel *>(Wg_c) + (size_t)r0 * d_model,
                                                     d_model);
        gather_rows_kernel<Tel><<<grid, 256, 0, s>>>(static_cast<const Tel *>(Wu), gather + r0,
                                                     static_cast<Tel *>(Wu_c) + (size_t)r0 * d_model,
                                                     d_model);
    }
    const int cx = ceil_div(n_rows, 256) < 64 ? ceil_div(n_rows, 256) : 64;
    for (int m0 = 0; m0 < d_model; m0 += 32768) {
        const int nm = d_model - m0 < 32768 ? d_model - m0 : 32768;
        dim3 grid(cx, nm);
        gather_cols_kernel<Tel><<<grid, 256, 0, s>>>(
            static_cast<const Tel *>(Wd) + (size_t)m0 * d_inter_src, gather,
            static_cast<Tel *>(Wd_c) + (size_t)m0 * n_rows, n_rows, d_inter_src);
    }
    return launch_status("gather kernels launch");
}

template <typename TIn, typename TH>
hipError_t launch_generic_typed(const FwdArgs &a, const BranchTable &bt)
{
    dim3 g1(ceil_div(a.d_inter, GT), ceil_div(a.T, GT));
    dim3 g2(ceil_div(a.d_model, GT), ceil_div(a.T, GT));
    if (g1.y > 65535u || g2.y > 65535u) return hipErrorInvalidValue;
    {
    ProfileScope ps(MLPMOE_KERNEL_GATE_UP_GENERIC, a.stream);
    gate_up_generic<TIn, TH><<<g1, GTHREADS, 0, a.stream>>>(
        static_cast<const TIn *>(a.x), static_cast<const TIn *>(a.Wg), static_cast<const TIn *>(a.Wu),
        static_cast<TH *>(a.H), a.T, a.d_model, a.d_inter, a.ldh, a.route, bt);
    }
    ProfileScope ps(MLPMOE_KERNEL_DOWN_GENERIC, a.stream);
    down_generic<TIn, TH><<<g2, GTHREADS, 0, a.stream>>>(
        static_cast<const TH *>(a.H), static_cast<const TIn *>(a.Wd), a.out, a.out_bf16 ? 1 : 0, a.T, a.d_model,
        a.d_inter, a.ldh, bt);
    return launch_status("generic kernels launch");
}

}  // namespace

hipError_t launch_fill_zero(float *out, size_t n, hipStream_t s)
{
    if (n == 0) return hipSuccess;
    size_t blocks = (n + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    ProfileScope ps(MLPMOE_KERNEL_FILL_ZERO, s);
    fill_zero_kernel<float><<<(unsigned)blocks, 256, 0, s>>>(out, n);
    return launch_status("fill_zero launch");
}

hipError_t launch_fill_zero16(uint16_t *out, size_t n, hipStream_t s)
{
    if (n == 0) return hipSuccess;
    size_t blocks = (n + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    ProfileScope ps(MLPMOE_KERNEL_FILL_ZERO, s);
    fill_zero_kernel<uint16_t><<<(unsigned)blocks, 256, 0, s>>>(out, n);
    return launch_status("fill_zero launch");
}

hipError_t launch_generic(const FwdArgs &a, const BranchTable &bt, bool is_bf16)
{
    return is_bf16 ? launch_generic_typed<uint16_t, uint16_t>(a, bt)
                   : launch_generic_typed<float, float>(a, bt);
}

hipError_t launch_compact(const void *Wg, const void *Wu, const void *Wd, const int32_t *gather,
                          int n_rows, int d_model, int d_inter_src, int elem_bytes, void *Wg_c,
                          void *Wu_c, void *Wd_c, hipStream_t s)
{
    return elem_bytes == 2
               ? compact_typed<uint16_t>(Wg, Wu, Wd, gather, n_rows, d_model, d_inter_src, Wg_c, Wu_c, Wd_c, s)
               : compact_typed<uint32_t>(Wg, Wu, Wd, gather, n_rows, d_model, d_inter_src, Wg_c, Wu_c, Wd_c, s);
}

}  // namespace mlpmoe
