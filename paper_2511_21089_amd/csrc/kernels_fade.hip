// Fractal Fade weight preparation (Sec. 3.2): for each branch with a sparsity ratio s > 0 and each
// of W_gate / W_up, zero the entries whose magnitude is not strictly greater than the
// linear-interpolation quantile of the block's magnitudes at fraction s.  bf16 storage first; float
// storage (two levels of the same histogram idea) further down.
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
#include <string.h>

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
        const unsigned long long add = (int)threadIdx.x >= d ? part[threadIdx.x - d] : 0;
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

// ---- float storage ----------------------------------------------------------------------------------
// A float magnitude is a 31-bit integer ordered like the value.  The order statistics at ranks
// floor(p) and floor(p) + 1 are found in two levels: a histogram of the upper 15 bits (the same
// 32768 bins in LDS) gives the bin of each rank and the rank's position inside its bin, a histogram of
// the lower 16 bits of the entries in those two bins (65536 bins each, global atomics: a bin holds a
// small share of the block) gives the rest of the bits.  The threshold is then interpolated on the host
// in double, exactly as the definition says, and fade_apply_f32 keeps the entries whose magnitude, as a
// double, is strictly greater; it counts the survivors as it goes.
constexpr int kLoBins = 65536;
constexpr int kSelWords = 8;      // per job, 64-bit: bin of rank 0, bin of rank 1, ranks inside those bins,
                                  // magnitude bits at rank 0, at rank 1, survivors, spare

__global__ void __launch_bounds__(kHistThreads)
fade_histogram_f32_hi(const uint32_t *__restrict__ W, uint32_t *__restrict__ hist, size_t hist_stride, FadeJobs jobs)
{
    extern __shared__ uint32_t lh[];                       // kBins counters
    const int j = blockIdx.y;
    for (int i = threadIdx.x; i < kBins; i += kHistThreads) lh[i] = 0;
    __syncthreads();
    const u32x4 *src = reinterpret_cast<const u32x4 *>(W + jobs.first[j]);
    const long long chunks = jobs.count[j] / 4;
    for (long long c = (long long)blockIdx.x * kHistThreads + threadIdx.x; c < chunks;
         c += (long long)gridDim.x * kHistThreads) {
        const u32x4 v = src[c];
#pragma unroll
        for (int q = 0; q < 4; ++q) atomicAdd(&lh[(v[q] & 0x7FFFFFFFu) >> 16], 1u);
    }
    __syncthreads();
    uint32_t *gh = hist + (size_t)j * hist_stride;
    for (int i = threadIdx.x; i < kBins; i += kHistThreads) {
        const uint32_t c = lh[i];
        if (c) atomicAdd(&gh[i], c);
    }
}

// Scans `bins` counters (a multiple of 1024) for the bins that hold ranks r0 and r1.  Every thread owns
// bins / 1024 consecutive bins; returns through the pointers (written by the owning thread only):
// the bin of each rank and the number of entries in the bins before it.
__device__ __forceinline__ void scan_for_ranks(const uint32_t *__restrict__ gh, int bins, unsigned long long r0,
                                               unsigned long long r1, unsigned long long *part,
                                               unsigned long long *out_bin0, unsigned long long *out_before0,
                                               unsigned long long *out_bin1, unsigned long long *out_before1)
{
    const int per = bins / 1024;
    unsigned long long mine = 0;
    for (int i = 0; i < per; ++i) mine += gh[threadIdx.x * per + i];
    part[threadIdx.x] = mine;
    __syncthreads();
    for (int d = 1; d < 1024; d <<= 1) {
        const unsigned long long add = (int)threadIdx.x >= d ? part[threadIdx.x - d] : 0;
        __syncthreads();
        part[threadIdx.x] += add;
        __syncthreads();
    }
    unsigned long long cum = part[threadIdx.x] - mine;
    for (int i = 0; i < per; ++i) {
        const int bin = threadIdx.x * per + i;
        const unsigned long long c = gh[bin];
        if (c) {
            if (r0 >= cum && r0 < cum + c) {
                *out_bin0 = (unsigned long long)bin;
                *out_before0 = cum;
            }
            if (r1 >= cum && r1 < cum + c) {
                *out_bin1 = (unsigned long long)bin;
                *out_before1 = cum;
            }
        }
        cum += c;
    }
    __syncthreads();
}

__global__ void __launch_bounds__(1024)
fade_select_f32_hi(const uint32_t *__restrict__ hist, size_t hist_stride, unsigned long long *__restrict__ sel,
                   FadeJobs jobs)
{
    __shared__ unsigned long long part[1024];
    __shared__ unsigned long long found[4];
    const int j = blockIdx.x;
    const unsigned long long total = (unsigned long long)jobs.count[j];
    const unsigned long long r0 = (unsigned long long)jobs.rank[j];
    const unsigned long long r1 = r0 + 1 < total ? r0 + 1 : total - 1;
    scan_for_ranks(hist + (size_t)j * hist_stride, kBins, r0, r1, part, &found[0], &found[1], &found[2], &found[3]);
    if (threadIdx.x == 0) {
        unsigned long long *o = sel + (size_t)j * kSelWords;
        o[0] = found[0];                 // upper 15 bits of the magnitude at rank r0
        o[1] = found[2];                 // ... at rank r1
        o[2] = r0 - found[1];            // position of rank r0 among the entries of its bin
        o[3] = r1 - found[3];
    }
}

__global__ void __launch_bounds__(256)
fade_histogram_f32_lo(const uint32_t *__restrict__ W, const unsigned long long *__restrict__ sel,
                      uint32_t *__restrict__ hist_lo, size_t hist_stride, FadeJobs jobs)
{
    const int j = blockIdx.y;
    const uint32_t bin0 = (uint32_t)sel[(size_t)j * kSelWords], bin1 = (uint32_t)sel[(size_t)j * kSelWords + 1];
    uint32_t *h0 = hist_lo + (size_t)j * hist_stride, *h1 = h0 + kLoBins;
    const u32x4 *src = reinterpret_cast<const u32x4 *>(W + jobs.first[j]);
    const long long chunks = jobs.count[j] / 4;
    for (long long c = (long long)blockIdx.x * 256 + threadIdx.x; c < chunks; c += (long long)gridDim.x * 256) {
        const u32x4 v = src[c];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint32_t m = v[q] & 0x7FFFFFFFu;
            if ((m >> 16) == bin0) atomicAdd(&h0[m & 0xFFFFu], 1u);
            if ((m >> 16) == bin1) atomicAdd(&h1[m & 0xFFFFu], 1u);
        }
    }
}

__global__ void __launch_bounds__(1024)
fade_select_f32_lo(const uint32_t *__restrict__ hist_lo, size_t hist_stride, unsigned long long *__restrict__ sel)
{
    __shared__ unsigned long long part[1024];
    __shared__ unsigned long long found[4];
    const int j = blockIdx.x;
    unsigned long long *o = sel + (size_t)j * kSelWords;
    const uint32_t *h0 = hist_lo + (size_t)j * hist_stride, *h1 = h0 + kLoBins;
    const unsigned long long never = ~0ULL;
    // rank r0 inside its bin, then rank r1 inside its own (the second rank of each scan is unused)
    scan_for_ranks(h0, kLoBins, o[2], never, part, &found[0], &found[1], &found[2], &found[3]);
    if (threadIdx.x == 0) o[4] = (o[0] << 16) | found[0];
    __syncthreads();
    scan_for_ranks(h1, kLoBins, o[3], never, part, &found[0], &found[1], &found[2], &found[3]);
    if (threadIdx.x == 0) o[5] = (o[1] << 16) | found[0];
}

struct FadeThresholds {
    double thr[MLPMOE_MAX_BRANCHES];
};

__global__ void __launch_bounds__(256)
fade_apply_f32(uint32_t *__restrict__ W, unsigned long long *__restrict__ sel, FadeThresholds th, FadeJobs jobs)
{
    const int j = blockIdx.y;
    const double thr = th.thr[j];
    u32x4 *dst = reinterpret_cast<u32x4 *>(W + jobs.first[j]);
    const long long chunks = jobs.count[j] / 4;
    unsigned long long kept = 0;
    for (long long c = (long long)blockIdx.x * 256 + threadIdx.x; c < chunks; c += (long long)gridDim.x * 256) {
        u32x4 v = dst[c];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const double a = (double)__uint_as_float(v[q] & 0x7FFFFFFFu);
            if (a > thr) ++kept;
            else v[q] &= 0x80000000u;                      // the entry times 0: the sign stays
        }
        dst[c] = v;
    }
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) kept += __shfl_xor(kept, d);
    if ((threadIdx.x & 63) == 0 && kept) atomicAdd(&sel[(size_t)j * kSelWords + 6], kept);
}

// ---- structured form: whole neurons ranked by the squared norm of their gate and up rows ----------
// One wave per neuron.  Squares of bf16 values are exact in double; every lane adds its share of the
// row in double, the lanes are added up by a butterfly (the order is fixed, the result the same in
// all lanes).  d_model is a multiple of 8 (bf16) or 4 (float).
template <bool kFloat>
__global__ void __launch_bounds__(256)
fade_neuron_scores(const void *__restrict__ Wg_, const void *__restrict__ Wu_, double *__restrict__ scores,
                   int d_inter, int d_model)
{
    const int lane = threadIdx.x & 63;
    const long long j = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (j >= d_inter) return;
    double acc = 0.0;
    if (kFloat) {
        // squares of floats are exact in double too (24 x 24 bits); d_model is a multiple of 4
        const float *g = static_cast<const float *>(Wg_) + (size_t)j * d_model;
        const float *u = static_cast<const float *>(Wu_) + (size_t)j * d_model;
        for (int k = lane * 4; k < d_model; k += 64 * 4) {
            const float4 a = *reinterpret_cast<const float4 *>(g + k);
            const float4 b = *reinterpret_cast<const float4 *>(u + k);
            const float w[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
            for (int i = 0; i < 8; ++i) acc += (double)w[i] * (double)w[i];
        }
    } else {
        const uint16_t *g = static_cast<const uint16_t *>(Wg_) + (size_t)j * d_model;
        const uint16_t *u = static_cast<const uint16_t *>(Wu_) + (size_t)j * d_model;
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
hipError_t launch_fade_neurons(const void *Wg, const void *Wu, const int32_t *off, const int32_t *keep_count,
                               int B, int d_model, int d_inter, int elem_bytes, double *scores, uint8_t *keep,
                               hipStream_t s)
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
    if (elem_bytes == 4)
        fade_neuron_scores<true><<<(unsigned)((d_inter + 3) / 4), 256, 0, s>>>(Wg, Wu, scores, d_inter, d_model);
    else
        fade_neuron_scores<false><<<(unsigned)((d_inter + 3) / 4), 256, 0, s>>>(Wg, Wu, scores, d_inter, d_model);
    if (launch_status("fade_neuron_scores launch") != hipSuccess) return hipErrorLaunchFailure;
    fade_neuron_select<<<dim3((unsigned)((widest + 255) / 256), (unsigned)B), 256, 0, s>>>(scores, keep, jobs);
    return launch_status("fade_neuron_select launch");
}

// The blocks of one projection matrix that are to be faded, and the rank floor(s (n - 1)) of each.
static void build_fade_jobs(const int32_t *off, const double *sparsity, int B, int d_model, FadeJobs &jobs,
                            int *job_of_branch)
{
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
}

// Per device, on the first call there: allow the 128 KB histogram in LDS.
template <typename K>
static hipError_t allow_big_histogram(K kernel, bool *attr_set, std::mutex &mu)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return note_hip_error("hipGetDevice", e);
    if (dev < 0 || dev >= 64) return note_hip_error("device index", hipErrorInvalidDevice);
    std::lock_guard<std::mutex> lock(mu);
    if (!attr_set[dev]) {
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                kBins * 4);
        if (e != hipSuccess) return note_hip_error("hipFuncSetAttribute(fade histogram)", e);
        attr_set[dev] = true;
    }
    return hipSuccess;
}

// Workgroups per block for the LDS histogram: enough to fill the chip, but at least ~16 chunks per thread
// so that the 128 KB histogram clear / flush of a workgroup is amortised.
static long long histogram_blocks(long long max_chunks, int n_jobs)
{
    long long per_block = (max_chunks + kHistThreads * 16 - 1) / (kHistThreads * 16);
    const long long want = (1024 + n_jobs - 1) / n_jobs;
    if (per_block > want) per_block = want;
    return per_block < 1 ? 1 : per_block;
}

// One projection matrix W [d_inter, d_model] (bf16, device).  off / sparsity are host arrays.
// scratch: device, >= B * (kBins + 4) uint32.  host_result: B * 4 uint32 (filled for faded branches).
// job_of_branch[b] = index into host_result / -1.
hipError_t launch_fade_bf16(void *W, const int32_t *off, const double *sparsity, int B, int d_model,
                            uint32_t *scratch, uint32_t *host_result, int *job_of_branch, hipStream_t s)
{
    FadeJobs jobs;
    build_fade_jobs(off, sparsity, B, d_model, jobs, job_of_branch);
    if (jobs.n == 0) return hipSuccess;
    uint32_t *hist = scratch;
    uint32_t *result = scratch + (size_t)jobs.n * kBins;
    const size_t words = (size_t)jobs.n * (kBins + 4);
    fill_u32<<<1024, 256, 0, s>>>(scratch, words);
    if (launch_status("fade fill launch") != hipSuccess) return hipErrorLaunchFailure;
    {
        static std::mutex mu;
        static bool attr_set[64] = {false};
        const hipError_t e = allow_big_histogram(&fade_histogram, attr_set, mu);
        if (e != hipSuccess) return e;
    }
    long long max_chunks = 0;
    for (int j = 0; j < jobs.n; ++j) max_chunks = jobs.count[j] / 8 > max_chunks ? jobs.count[j] / 8 : max_chunks;
    fade_histogram<<<dim3((unsigned)histogram_blocks(max_chunks, jobs.n), (unsigned)jobs.n), kHistThreads, kBins * 4, s>>>(
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

// Float storage.  scratch: device, >= fade_scratch_words_f32(B) uint32.  On return thresholds[j] (double) and
// kept[j] are filled for every job; job_of_branch as above.  Synchronises the stream twice: once to read the
// two order statistics back (the threshold is interpolated on the host, in double, from exactly those two
// numbers), once at the end.
hipError_t launch_fade_f32(void *W, const int32_t *off, const double *sparsity, int B, int d_model,
                           uint32_t *scratch, double *thresholds, long long *kept, int *job_of_branch, hipStream_t s)
{
    FadeJobs jobs;
    build_fade_jobs(off, sparsity, B, d_model, jobs, job_of_branch);
    if (jobs.n == 0) return hipSuccess;
    // per job: upper histogram, two lower histograms, the select words (64-bit, 8-byte aligned: even word counts)
    const size_t hist_words = (size_t)kBins + 2 * (size_t)kLoBins;
    uint32_t *hist = scratch;
    unsigned long long *sel = reinterpret_cast<unsigned long long *>(scratch + (size_t)jobs.n * hist_words);
    const size_t words = (size_t)jobs.n * (hist_words + 2 * kSelWords);
    fill_u32<<<2048, 256, 0, s>>>(scratch, words);
    if (launch_status("fade fill launch") != hipSuccess) return hipErrorLaunchFailure;
    {
        static std::mutex mu;
        static bool attr_set[64] = {false};
        const hipError_t e = allow_big_histogram(&fade_histogram_f32_hi, attr_set, mu);
        if (e != hipSuccess) return e;
    }
    long long max_chunks = 0;
    for (int j = 0; j < jobs.n; ++j) max_chunks = jobs.count[j] / 4 > max_chunks ? jobs.count[j] / 4 : max_chunks;
    const uint32_t *Wc = static_cast<const uint32_t *>(W);
    fade_histogram_f32_hi<<<dim3((unsigned)histogram_blocks(max_chunks, jobs.n), (unsigned)jobs.n), kHistThreads,
                            kBins * 4, s>>>(Wc, hist, hist_words, jobs);
    if (launch_status("fade_histogram_f32_hi launch") != hipSuccess) return hipErrorLaunchFailure;
    fade_select_f32_hi<<<jobs.n, 1024, 0, s>>>(hist, hist_words, sel, jobs);
    if (launch_status("fade_select_f32_hi launch") != hipSuccess) return hipErrorLaunchFailure;
    long long blocks = (max_chunks + 256 * 8 - 1) / (256 * 8);
    if (blocks > 2048) blocks = 2048;
    if (blocks < 1) blocks = 1;
    fade_histogram_f32_lo<<<dim3((unsigned)blocks, (unsigned)jobs.n), 256, 0, s>>>(Wc, sel, hist + kBins, hist_words, jobs);
    if (launch_status("fade_histogram_f32_lo launch") != hipSuccess) return hipErrorLaunchFailure;
    fade_select_f32_lo<<<jobs.n, 1024, 0, s>>>(hist + kBins, hist_words, sel);
    if (launch_status("fade_select_f32_lo launch") != hipSuccess) return hipErrorLaunchFailure;
    unsigned long long host_sel[MLPMOE_MAX_BRANCHES * kSelWords];
    const size_t sel_bytes = (size_t)jobs.n * kSelWords * sizeof(unsigned long long);
    hipError_t e = hipMemcpyAsync(host_sel, sel, sel_bytes, hipMemcpyDeviceToHost, s);
    if (e != hipSuccess) return note_hip_error("hipMemcpyAsync(fade order statistics)", e);
    e = hipStreamSynchronize(s);
    if (e != hipSuccess) return note_hip_error("hipStreamSynchronize(fade)", e);
    FadeThresholds th;
    for (int b = 0; b < B; ++b) {
        const int j = job_of_branch[b];
        if (j < 0) continue;
        const double p = sparsity[b] * (double)(jobs.count[j] - 1);
        const double frac = p - (double)(long long)p;
        const uint32_t lo_bits = (uint32_t)host_sel[(size_t)j * kSelWords + 4];
        const uint32_t hi_bits = (uint32_t)host_sel[(size_t)j * kSelWords + 5];
        float lo, hi;
        memcpy(&lo, &lo_bits, 4);
        memcpy(&hi, &hi_bits, 4);
        // two roundings, product then sum, as the definition's double arithmetic has them
        volatile double step = frac * ((double)hi - (double)lo);
        th.thr[j] = (double)lo + step;
        thresholds[j] = th.thr[j];
    }
    fade_apply_f32<<<dim3((unsigned)blocks, (unsigned)jobs.n), 256, 0, s>>>(static_cast<uint32_t *>(W), sel, th, jobs);
    if (launch_status("fade_apply_f32 launch") != hipSuccess) return hipErrorLaunchFailure;
    e = hipMemcpyAsync(host_sel, sel, sel_bytes, hipMemcpyDeviceToHost, s);
    if (e != hipSuccess) return note_hip_error("hipMemcpyAsync(fade survivors)", e);
    e = hipStreamSynchronize(s);
    if (e != hipSuccess) return note_hip_error("hipStreamSynchronize(fade)", e);
    for (int j = 0; j < jobs.n; ++j) kept[j] = (long long)host_sel[(size_t)j * kSelWords + 6];
    return hipSuccess;
}

size_t fade_scratch_words_f32(int B) { return (size_t)B * ((size_t)kBins + 2 * (size_t)kLoBins + 2 * kSelWords); }

}  // namespace mlpmoe
