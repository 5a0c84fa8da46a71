// Fractal Fade weight preparation (Sec. 3.2) for bf16 weights: for each branch with a sparsity
// ratio s > 0 and each of W_gate / W_up, zero the entries whose magnitude is not strictly greater
// than the linear-interpolation quantile of the block's magnitudes at fraction s.
//
// A bf16 magnitude is a 15-bit integer whose order is the order of the values, so the order
// statistics of a block are read off an exact histogram with 32768 bins:
//   1. fade_histogram: every workgroup counts its share of a block in an LDS histogram (128 KB)
//      and adds the non-empty bins to the block's histogram in global memory;
//   2. fade_select: one workgroup per block scans the bins for the order statistics at ranks
//      floor(p) and floor(p) + 1, p = s (n - 1), and counts the survivors;
//   3. fade_apply: entries with magnitude <= the order statistic at floor(p) keep only their sign
//      bit (the value times 0).
// Between two neighbouring order statistics there is no data, so "greater than the interpolated
// threshold" and "greater than the lower neighbour" select the same entries; the interpolated
// value itself is formed on the host from the two neighbours, for reporting.
#include <mutex>

#include "internal.h"

namespace mlpmoe {
namespace {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int kBins = 32768;
constexpr int kHistThreads = 512;

struct FadeJobs {
    int n;                       // blocks to process (<= MLPMOE_MAX_BRANCHES)
    long long first[MLPMOE_MAX_BRANCHES];   // first element of the block in the weight matrix
    long long count[MLPMOE_MAX_BRANCHES];   // elements in the block (a multiple of 8)
    long long rank[MLPMOE_MAX_BRANCHES];    // floor(s (count - 1))
};

__global__ void __launch_bounds__(kHistThreads)
fade_histogram(const uint16_t *__restrict__ W, uint32_t *__restrict__ hist, FadeJobs jobs)
{
    extern __shared__ uint32_t lh[];                       // kBins counters
    const int j = blockIdx.y;
    for (int i = threadIdx.x; i < kBins; i += kHistThreads) lh[i] = 0;
    __syncthreads();
    const u32x4 *src = reinterpret_cast<const u32x4 *>(W + jobs.first[j]);
    const long long chunks = jobs.count[j] / 8;
    for (long long c = (long long)blockIdx.x * kHistThreads + threadIdx.x; c < chunks;
         c += (long long)gridDim.x * kHistThreads) {
        const u32x4 v = src[c];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            atomicAdd(&lh[v[q] & 0x7FFFu], 1u);
            atomicAdd(&lh[(v[q] >> 16) & 0x7FFFu], 1u);
        }
    }
    __syncthreads();
    uint32_t *gh = hist + (size_t)j * kBins;
    for (int i = threadIdx.x; i < kBins; i += kHistThreads) {
        const uint32_t c = lh[i];
        if (c) atomicAdd(&gh[i], c);
    }
}

// result[j] = {magnitude bits at rank floor(p), magnitude bits at rank floor(p)+1 (clamped to the
// last element), survivors low word, survivors high word}
__global__ void __launch_bounds__(1024)
fade_select(const uint32_t *__restrict__ hist, uint32_t *__restrict__ result, FadeJobs jobs)
{
    __shared__ unsigned long long part[1024];
    const int j = blockIdx.x;
    const uint32_t *gh = hist + (size_t)j * kBins;
    constexpr int per = kBins / 1024;                      // 32 consecutive bins per thread
    unsigned long long mine = 0;
    for (int i = 0; i < per; ++i) mine += gh[threadIdx.x * per + i];
    part[threadIdx.x] = mine;
    __syncthreads();
    // inclusive scan over the 1024 partial sums
    for (int d = 1; d < 1024; d <<= 1) {
        const unsigned long long add = threadIdx.x >= d ? part[threadIdx.x - d] : 0;
        __syncthreads();
        part[threadIdx.x] += add;
        __syncthreads();
    }
    const unsigned long long before = part[threadIdx.x] - mine;     // elements in earlier bins
    const unsigned long long total = part[1023];
    const unsigned long long r0 = (unsigned long long)jobs.rank[j];
    const unsigned long long r1 = r0 + 1 < total ? r0 + 1 : total - 1;
    unsigned long long cum = before;
    for (int i = 0; i < per; ++i) {
        const int bin = threadIdx.x * per + i;
        const unsigned long long c = gh[bin];
        if (c) {
            if (r0 >= cum && r0 < cum + c) {
                result[4 * j] = (uint32_t)bin;
                const unsigned long long kept = total - (cum + c);
                result[4 * j + 2] = (uint32_t)kept;
                result[4 * j + 3] = (uint32_t)(kept >> 32);
            }
            if (r1 >= cum && r1 < cum + c) result[4 * j + 1] = (uint32_t)bin;
        }
        cum += c;
    }
}

__global__ void __launch_bounds__(256)
fade_apply(uint16_t *__restrict__ W, const uint32_t *__restrict__ result, FadeJobs jobs)
{
    const int j = blockIdx.y;
    const uint32_t cut = result[4 * j];                    // magnitudes <= cut are zeroed
    u32x4 *dst = reinterpret_cast<u32x4 *>(W + jobs.first[j]);
    const long long chunks = jobs.count[j] / 8;
    for (long long c = (long long)blockIdx.x * 256 + threadIdx.x; c < chunks; c += (long long)gridDim.x * 256) {
        u32x4 v = dst[c];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            uint32_t lo = v[q] & 0xFFFFu, hi = v[q] >> 16;
            if ((lo & 0x7FFFu) <= cut) lo &= 0x8000u;
            if ((hi & 0x7FFFu) <= cut) hi &= 0x8000u;
            v[q] = lo | (hi << 16);
        }
        dst[c] = v;
    }
}

__global__ void fill_u32(uint32_t *p, size_t n)
{
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
        p[i] = 0;
}

// ---- structured form: whole neurons ranked by the squared norm of their gate and up rows ----------
// One wave per neuron.  Squares of bf16 values are exact in double; every lane adds its share of the
// row in double, the lanes are added up by a butterfly (the order is fixed, the result the same in
// all lanes).  d_model is a multiple of 8.
__global__ void __launch_bounds__(256)
fade_neuron_scores(const uint16_t *__restrict__ Wg, const uint16_t *__restrict__ Wu, double *__restrict__ scores,
                   int d_inter, int d_model)
{
    const int lane = threadIdx.x & 63;
    const long long j = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (j >= d_inter) return;
    const uint16_t *g = Wg + (size_t)j * d_model, *u = Wu + (size_t)j * d_model;
    double acc = 0.0;
    for (int k = lane * 8; k < d_model; k += 64 * 8) {
        const uint4 a = *reinterpret_cast<const uint4 *>(g + k);
        const uint4 b = *reinterpret_cast<const uint4 *>(u + k);
        const uint32_t w[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const double lo = (double)__uint_as_float(w[i] << 16), hi = (double)__uint_as_float(w[i] & 0xffff0000u);
            acc += lo * lo;
            acc += hi * hi;
        }
    }
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) acc += __shfl_xor(acc, d);
    if (lane == 0) scores[j] = acc;
}

struct NeuronJobs {
    int B;
    int off[MLPMOE_MAX_BRANCHES + 1];
    int keep[MLPMOE_MAX_BRANCHES];
};

// keep[j] = 1 if fewer than keep_count[b] neurons of j's branch come before it (larger score, or the
// same score and a lower index).  One thread per neuron, grid.y = branch.
__global__ void __launch_bounds__(256)
fade_neuron_select(const double *__restrict__ scores, uint8_t *__restrict__ keep, NeuronJobs jobs)
{
    const int b = blockIdx.y;
    const int lo = jobs.off[b], hi = jobs.off[b + 1];
    const int j = lo + blockIdx.x * 256 + threadIdx.x;
    if (j >= hi) return;
    const double mine = scores[j];
    int before = 0;
    for (int i = lo; i < hi; ++i) {
        const double other = scores[i];                    // the same address in every lane: one broadcast read
        before += (other > mine || (other == mine && i < j)) ? 1 : 0;
    }
    keep[j] = before < jobs.keep[b] ? 1 : 0;
}

}  // namespace

// Structured fade: scores (device, d_inter doubles) and keep flags (device, d_inter bytes) of all neurons.
// off / keep_count are host arrays (validated by the caller).  Asynchronous on s.
hipError_t launch_fade_neurons_bf16(const void *Wg, const void *Wu, const int32_t *off, const int32_t *keep_count,
                                    int B, int d_model, int d_inter, double *scores, uint8_t *keep, hipStream_t s)
{
    if (d_inter == 0) return hipSuccess;
    NeuronJobs jobs;
    jobs.B = B;
    int widest = 0;
    for (int b = 0; b < B; ++b) {
        jobs.off[b] = off[b];
        jobs.keep[b] = keep_count[b];
        widest = off[b + 1] - off[b] > widest ? off[b + 1] - off[b] : widest;
    }
    jobs.off[B] = off[B];
    fade_neuron_scores<<<(unsigned)((d_inter + 3) / 4), 256, 0, s>>>(
        static_cast<const uint16_t *>(Wg), static_cast<const uint16_t *>(Wu), scores, d_inter, d_model);
    if (launch_status("fade_neuron_scores launch") != hipSuccess) return hipErrorLaunchFailure;
    fade_neuron_select<<<dim3((unsigned)((widest + 255) / 256), (unsigned)B), 256, 0, s>>>(scores, keep, jobs);
    return launch_status("fade_neuron_select launch");
}

// One projection matrix W [d_inter, d_model] (bf16, device).  off / sparsity are host arrays.
// scratch: device, >= B * (kBins + 4) uint32.  host_result: B * 4 uint32 (filled for faded branches).
// job_of_branch[b] = index into host_result / -1.
hipError_t launch_fade_bf16(void *W, const int32_t *off, const double *sparsity, int B, int d_model,
                            uint32_t *scratch, uint32_t *host_result, int *job_of_branch, hipStream_t s)
{
    FadeJobs jobs;
    jobs.n = 0;
    for (int b = 0; b < B; ++b) {
        job_of_branch[b] = -1;
        const long long n = (long long)(off[b + 1] - off[b]) * d_model;
        if (!(sparsity[b] > 0.0) || n == 0) continue;
        const int j = jobs.n++;
        job_of_branch[b] = j;
        jobs.first[j] = (long long)off[b] * d_model;
        jobs.count[j] = n;
        const double p = sparsity[b] * (double)(n - 1);
        long long r = (long long)p;                        // p >= 0: truncation is floor
        if (r > n - 1) r = n - 1;
        jobs.rank[j] = r;
    }
    if (jobs.n == 0) return hipSuccess;
    uint32_t *hist = scratch;
    uint32_t *result = scratch + (size_t)jobs.n * kBins;
    const size_t words = (size_t)jobs.n * (kBins + 4);
    fill_u32<<<1024, 256, 0, s>>>(scratch, words);
    if (launch_status("fade fill launch") != hipSuccess) return hipErrorLaunchFailure;
    {
        // per device, on the first call there: allow the 128 KB histogram
        static std::mutex mu;
        static bool attr_set[64] = {false};
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return note_hip_error("hipGetDevice", e);
        if (dev < 0 || dev >= 64) return note_hip_error("device index", hipErrorInvalidDevice);
        std::lock_guard<std::mutex> lock(mu);
        if (!attr_set[dev]) {
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(&fade_histogram),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, kBins * 4);
            if (e != hipSuccess) return note_hip_error("hipFuncSetAttribute(fade_histogram)", e);
            attr_set[dev] = true;
        }
    }
    long long max_chunks = 0;
    for (int j = 0; j < jobs.n; ++j) max_chunks = jobs.count[j] / 8 > max_chunks ? jobs.count[j] / 8 : max_chunks;
    // enough workgroups per block to fill the chip, but at least ~16 chunks per thread so that the
    // 128 KB histogram clear / flush of a workgroup is amortised
    long long per_block = (max_chunks + kHistThreads * 16 - 1) / (kHistThreads * 16);
    const long long want = (1024 + jobs.n - 1) / jobs.n;
    if (per_block > want) per_block = want;
    if (per_block < 1) per_block = 1;
    fade_histogram<<<dim3((unsigned)per_block, (unsigned)jobs.n), kHistThreads, kBins * 4, s>>>(
        static_cast<const uint16_t *>(W), hist, jobs);
    if (launch_status("fade_histogram launch") != hipSuccess) return hipErrorLaunchFailure;
    fade_select<<<jobs.n, 1024, 0, s>>>(hist, result, jobs);
    if (launch_status("fade_select launch") != hipSuccess) return hipErrorLaunchFailure;
    long long apply_blocks = (max_chunks + 256 * 8 - 1) / (256 * 8);
    if (apply_blocks > 2048) apply_blocks = 2048;
    if (apply_blocks < 1) apply_blocks = 1;
    fade_apply<<<dim3((unsigned)apply_blocks, (unsigned)jobs.n), 256, 0, s>>>(static_cast<uint16_t *>(W), result, jobs);
    if (launch_status("fade_apply launch") != hipSuccess) return hipErrorLaunchFailure;
    hipError_t e = hipMemcpyAsync(host_result, result, (size_t)jobs.n * 4 * sizeof(uint32_t), hipMemcpyDeviceToHost, s);
    if (e != hipSuccess) return note_hip_error("hipMemcpyAsync(fade result)", e);
    e = hipStreamSynchronize(s);
    if (e != hipSuccess) return note_hip_error("hipStreamSynchronize(fade)", e);
    return hipSuccess;
}

size_t fade_scratch_words(int B) { return (size_t)B * (kBins + 4); }

}  // namespace mlpmoe
