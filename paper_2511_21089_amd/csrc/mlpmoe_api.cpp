// Host side of the C ABI: argument validation, the slicing rules, the branch
// table, workspace management and kernel-path dispatch.  No arithmetic of the
// forward itself lives here.
#include <math.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <map>
#include <mutex>
#include <new>
#include <vector>

#include "internal.h"

using namespace mlpmoe;

namespace {

struct DeviceWorkspace {
    void *ptr = nullptr;          // library-owned block (hipMalloc), grown on demand
    size_t bytes = 0;
    void *user_ptr = nullptr;     // caller's block (mlpmoe_set_workspace); when set, nothing is ever allocated
    size_t user_bytes = 0;
};
// Guards g_ws and, for the entry points without a workspace argument, stays locked from the moment
// the block is chosen until the kernels that use it are enqueued: a growth on another thread
// synchronises the device before it frees, so work already enqueued is never left with a freed block.
std::mutex g_ws_mutex;
std::map<int, DeviceWorkspace> g_ws;

// Scratch of mlpmoe_forward_bf16_noalloc: device memory that exists from the moment the code
// object is loaded, one copy per GPU.  Host code never uses this name as an address; it asks the
// runtime for the device address once per device (noalloc_scratch) and passes that to the kernels.
static __device__ __align__(256) unsigned char g_noalloc_scratch[MLPMOE_NOALLOC_SCRATCH_BYTES];

// --- per-kernel event timing -------------------------------------------------
struct Profiler {
    bool on = false;
    int capacity = 0, count = 0;
    std::vector<hipEvent_t> ev;      // 2 per record: begin, end
    std::vector<int> ids;
} g_prof;

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int validate_common(const void *x, const void *Wg, const void *Wu, const void *Wd,
                    const int32_t *off, const float *alpha, const uint8_t *mask, int T, int d_model,
                    int d_inter, int B, const float *out)
{
    if (!off || !alpha || !mask) return MLPMOE_ERR_NULL;
    if (B < 1 || B > MLPMOE_MAX_BRANCHES || T < 0 || d_model < 1 || d_inter < 0)
        return MLPMOE_ERR_SHAPE;
    // index arithmetic inside the kernels is 32-bit for rows and columns, 64-bit for addresses; byte
    // offsets of a row inside a 256-row tile (row * leading dimension * 2) are 32-bit unsigned, which
    // bounds the leading dimensions d_model and d_inter (+63 for the intermediate) by 2^22
    if ((long long)T * d_model > (1LL << 40) || (long long)d_inter * d_model > (1LL << 40) ||
        d_model > (1 << 22) || d_inter > (1 << 22) || T > (1 << 24))
        return MLPMOE_ERR_SHAPE;
    if (off[0] != 0) return MLPMOE_ERR_OFFSETS;
    for (int b = 0; b < B; ++b)
        if (off[b + 1] < off[b]) return MLPMOE_ERR_OFFSETS;
    if (off[B] != d_inter) return MLPMOE_ERR_OFFSETS;
    if (T == 0) return MLPMOE_OK;
    if (!x || !out) return MLPMOE_ERR_NULL;
    if (d_inter > 0 && (!Wg || !Wu || !Wd)) return MLPMOE_ERR_NULL;
    if (!aligned16(x) || !aligned16(out) || !aligned16(Wg) || !aligned16(Wu) || !aligned16(Wd))
        return MLPMOE_ERR_ALIGN;
    return MLPMOE_OK;
}

void build_table(const int32_t *off, const float *alpha, const uint8_t *mask, int B, BranchTable &bt)
{
    memset(&bt, 0, sizeof(bt));
    bt.B = B;
    for (int b = 0; b <= B; ++b) bt.off[b] = off[b];
    int runs = 0;
    for (int b = 0; b < B; ++b) {
        bt.alpha[b] = alpha[b];
        if (!mask[b]) continue;
        bt.active |= 1ULL << b;
        if (off[b + 1] == off[b]) continue;
        bt.d_eff += off[b + 1] - off[b];
        if (runs > 0 && bt.run_end[runs - 1] == off[b]) {
            bt.run_end[runs - 1] = off[b + 1];
        } else {
            bt.run_start[runs] = off[b];
            bt.run_end[runs] = off[b + 1];
            ++runs;
        }
    }
    bt.n_runs = runs;
}

bool fast_path_aligned(const BranchTable &bt, int d_model, int d_inter)
{
    if (d_model % 8 != 0 || d_inter % 8 != 0) return false;
    for (int r = 0; r < bt.n_runs; ++r)
        if (bt.run_start[r] % 8 != 0 || bt.run_end[r] % 8 != 0) return false;
    return true;
}

size_t h_bytes(int T, int d_inter, int elem_bytes)
{
    return align_up((size_t)T * (size_t)h_ld(d_inter) * (size_t)elem_bytes, 256);
}

// Dispatch with a ready branch table: path choice, workspace carving, launch.  No loops over
// branches, no allocation, no synchronisation.
// route: per-token routing [T, B] on the device, or nullptr.  Routed calls use the kernels that skip
// (token tile, branch) pairs nobody is routed to when every branch boundary is a multiple of 8,
// and the generic kernels (masking only) otherwise.
int forward_table(const BranchTable &bt, bool aligned, const void *x, const void *Wg, const void *Wu,
                  const void *Wd, int T, int d_model, int d_inter, float *out, void *workspace,
                  size_t workspace_bytes, int path, bool is_bf16, hipStream_t stream,
                  const uint8_t *route = nullptr, bool out_bf16 = false)
{
    // launch status is read back with hipGetLastError(): drop whatever an earlier, unrelated
    // runtime call of this thread left behind (e.g. a "not ready" from an event query)
    (void)hipGetLastError();
    g_err_detail[0] = 0;

    if (bt.n_runs == 0) {   // nothing active: the sum over branches is empty
        const size_t n = (size_t)T * d_model;
        const hipError_t e = out_bf16 ? launch_fill_zero16(reinterpret_cast<uint16_t *>(out), n, stream)
                                      : launch_fill_zero(out, n, stream);
        return e == hipSuccess ? MLPMOE_OK : MLPMOE_ERR_HIP;
    }
    if (route) {
        // the routed K loops start and stop at branch boundaries, not only at run boundaries
        for (int b = 0; b <= bt.B && aligned; ++b) aligned = bt.off[b] % 8 == 0;
    }
    if (path == MLPMOE_PATH_AUTO)
        path = !aligned ? MLPMOE_PATH_GENERIC : (T <= 16 ? MLPMOE_PATH_DECODE : MLPMOE_PATH_MFMA);
    int tile_shape = -1;
    if (path >= MLPMOE_PATH_MFMA_WIDE && path <= MLPMOE_PATH_MFMA_SLIM) {
        tile_shape = path - MLPMOE_PATH_MFMA_WIDE;
        path = MLPMOE_PATH_MFMA;
        if (route && tile_shape >= 2) return MLPMOE_ERR_UNSUPPORTED;     // routed: 256-token tiles of one width
    }
    if (path != MLPMOE_PATH_GENERIC && !aligned) return MLPMOE_ERR_UNSUPPORTED;
    if (path == MLPMOE_PATH_DECODE && T > 16) return MLPMOE_ERR_UNSUPPORTED;

    const int elem = is_bf16 ? 2 : 4;
    const size_t need = mlpmoe_workspace_bytes(T, d_model, d_inter, bt.B, elem);
    if (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 255u))
        return MLPMOE_ERR_WORKSPACE;

    FwdArgs a;
    a.x = x; a.Wg = Wg; a.Wu = Wu; a.Wd = Wd; a.out = out;
    a.out_bf16 = out_bf16;
    a.T = T; a.d_model = d_model; a.d_inter = d_inter;
    a.H = workspace;
    a.ldh = h_ld(d_inter);
    a.partial_bytes = need - h_bytes(T, d_inter, elem) - route_scratch_bytes(T, d_inter) - 256;
    a.partial = a.partial_bytes
                    ? reinterpret_cast<float *>(static_cast<char *>(workspace) + h_bytes(T, d_inter, elem))
                    : nullptr;
    a.stream = stream;
    a.tile_shape = tile_shape;
    a.route = route;
    a.route_scratch = reinterpret_cast<uint8_t *>(static_cast<char *>(workspace) + need - route_scratch_bytes(T, d_inter));

    hipError_t e;
    if (path == MLPMOE_PATH_GENERIC) {
        e = launch_generic(a, bt, is_bf16);
    } else if (route) {
        e = path == MLPMOE_PATH_MFMA ? launch_mfma_routed_bf16(a, bt) : launch_decode_routed_bf16(a, bt);
    } else if (path == MLPMOE_PATH_MFMA) {
        e = launch_mfma_bf16(a, bt);
    } else {
        e = launch_decode_bf16(a, bt);
    }
    if (e != hipSuccess && g_err_detail[0] == 0) (void)note_hip_error("kernel launch", e);
    return e == hipSuccess ? MLPMOE_OK : MLPMOE_ERR_HIP;
}

int forward_impl(const void *x, const void *Wg, const void *Wu, const void *Wd, const int32_t *off,
                 const float *alpha, const uint8_t *mask, int T, int d_model, int d_inter, int B,
                 float *out, void *workspace, size_t workspace_bytes, int path, bool is_bf16,
                 hipStream_t stream, bool out_bf16 = false)
{
    int rc = validate_common(x, Wg, Wu, Wd, off, alpha, mask, T, d_model, d_inter, B, out);
    if (rc != MLPMOE_OK) return rc;
    if (path < MLPMOE_PATH_AUTO || path > MLPMOE_PATH_MFMA_SLIM) return MLPMOE_ERR_UNSUPPORTED;
    if (T == 0) return MLPMOE_OK;
    BranchTable bt;
    build_table(off, alpha, mask, B, bt);
    const bool aligned = is_bf16 && fast_path_aligned(bt, d_model, d_inter);
    return forward_table(bt, aligned, x, Wg, Wu, Wd, T, d_model, d_inter, out, workspace, workspace_bytes,
                         path, is_bf16, stream, nullptr, out_bf16);
}

// Workspace of the current device for the entry points that take none: the caller's block if one
// was set, else the library-owned one, grown on demand.  g_ws_mutex must be held by the caller.
int owned_workspace(size_t need, hipStream_t stream, void **ptr, size_t *bytes)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) {
        (void)note_hip_error("hipGetDevice", e);
        return MLPMOE_ERR_HIP;
    }
    DeviceWorkspace &w = g_ws[dev];
    if (w.user_ptr) {                        // caller-owned: use it or refuse, never allocate
        if (w.user_bytes < need) return MLPMOE_ERR_WORKSPACE;
        *ptr = w.user_ptr;
        *bytes = w.user_bytes;
        return MLPMOE_OK;
    }
    if (w.bytes < need) {
        // growing synchronises the device and allocates: neither is allowed while the stream records a graph
        hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
        if (hipStreamIsCapturing(stream, &cap) != hipSuccess) (void)hipGetLastError();
        if (cap != hipStreamCaptureStatusNone) return MLPMOE_ERR_WORKSPACE;
        if (w.ptr) {
            e = hipDeviceSynchronize();      // earlier launches may still be using the old block
            if (e != hipSuccess) {
                (void)note_hip_error("hipDeviceSynchronize before growing the workspace", e);
                return MLPMOE_ERR_HIP;
            }
            (void)hipFree(w.ptr);
            w.ptr = nullptr;
            w.bytes = 0;
        }
        void *p = nullptr;
        if (hipMalloc(&p, need) != hipSuccess) {
            (void)hipGetLastError();
            return MLPMOE_ERR_WORKSPACE;
        }
        w.ptr = p;
        w.bytes = need;
    }
    *ptr = w.ptr;
    *bytes = w.bytes;
    return MLPMOE_OK;
}

int forward_owned(const void *x, const void *Wg, const void *Wu, const void *Wd, const int32_t *off,
                  const float *alpha, const uint8_t *mask, int T, int d_model, int d_inter, int B,
                  float *out, bool is_bf16, hipStream_t stream, bool out_bf16 = false)
{
    int rc = validate_common(x, Wg, Wu, Wd, off, alpha, mask, T, d_model, d_inter, B, out);
    if (rc != MLPMOE_OK) return rc;
    if (T == 0) return MLPMOE_OK;
    size_t need = mlpmoe_workspace_bytes(T, d_model, d_inter, B, is_bf16 ? 2 : 4);
    void *ws = nullptr;
    size_t ws_bytes = 0;
    std::lock_guard<std::mutex> lock(g_ws_mutex);      // held until the kernels are enqueued
    rc = owned_workspace(need, stream, &ws, &ws_bytes);
    if (rc != MLPMOE_OK) return rc;
    return forward_impl(x, Wg, Wu, Wd, off, alpha, mask, T, d_model, d_inter, B, out, ws, ws_bytes,
                        MLPMOE_PATH_AUTO, is_bf16, stream, out_bf16);
}

// Device address of this GPU's copy of g_noalloc_scratch, asked from the runtime on the first call
// on each device (with that device current) and kept.
int noalloc_scratch(void **ptr)
{
    static std::mutex mu;
    static void *addr[64] = {nullptr};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) {
        (void)note_hip_error("hipGetDevice", e);
        return MLPMOE_ERR_HIP;
    }
    if (dev < 0 || dev >= 64) {
        (void)note_hip_error("device index", hipErrorInvalidDevice);
        return MLPMOE_ERR_HIP;
    }
    std::lock_guard<std::mutex> lock(mu);
    if (!addr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(g_noalloc_scratch));
        if (e != hipSuccess || !p) {
            (void)note_hip_error("hipGetSymbolAddress(noalloc scratch)", e);
            (void)hipGetLastError();
            return MLPMOE_ERR_HIP;
        }
        addr[dev] = p;
    }
    *ptr = addr[dev];
    return MLPMOE_OK;
}

}  // namespace

namespace mlpmoe {
thread_local char g_err_detail[192] = "";

hipError_t note_hip_error(const char *where, hipError_t e)
{
    snprintf(g_err_detail, sizeof(g_err_detail), "%s: %s", where, hipGetErrorString(e));
    return e;
}

void profile_mark(int kernel_id, hipStream_t s, bool begin)
{
    if (!g_prof.on) return;
    if (begin) {
        if (g_prof.count >= g_prof.capacity) return;
        g_prof.ids[g_prof.count] = kernel_id;
        (void)hipEventRecord(g_prof.ev[2 * g_prof.count], s);
    } else {
        if (g_prof.count >= g_prof.capacity) return;
        (void)hipEventRecord(g_prof.ev[2 * g_prof.count + 1], s);
        ++g_prof.count;
    }
}
}  // namespace mlpmoe

extern "C" {

int mlpmoe_profile_disable(void)
{
    for (hipEvent_t e : g_prof.ev) (void)hipEventDestroy(e);
    g_prof = Profiler();
    return MLPMOE_OK;
}

int mlpmoe_profile_enable(int capacity)
{
    if (capacity < 1 || capacity > 65536) return MLPMOE_ERR_SHAPE;
    mlpmoe_profile_disable();
    g_prof.ev.resize(2 * (size_t)capacity);
    g_prof.ids.assign(capacity, 0);
    for (size_t i = 0; i < g_prof.ev.size(); ++i)
        if (hipEventCreate(&g_prof.ev[i]) != hipSuccess) {
            g_prof.ev.resize(i);
            mlpmoe_profile_disable();
            return MLPMOE_ERR_HIP;
        }
    g_prof.capacity = capacity;
    g_prof.on = true;
    return MLPMOE_OK;
}

int mlpmoe_profile_collect(int *ids, float *ms, int capacity)
{
    if (!ids || !ms) return MLPMOE_ERR_NULL;
    if (capacity < 0) return MLPMOE_ERR_SHAPE;
    int n = g_prof.count < capacity ? g_prof.count : capacity;
    for (int i = 0; i < n; ++i) {
        if (hipEventSynchronize(g_prof.ev[2 * i + 1]) != hipSuccess ||
            hipEventElapsedTime(&ms[i], g_prof.ev[2 * i], g_prof.ev[2 * i + 1]) != hipSuccess)
            return MLPMOE_ERR_HIP;
        ids[i] = g_prof.ids[i];
    }
    g_prof.count = 0;
    return n;
}

const char *mlpmoe_last_error_detail(void) { return mlpmoe::g_err_detail; }

const char *mlpmoe_status_string(int status)
{
    switch (status) {
    case MLPMOE_OK: return "ok";
    case MLPMOE_ERR_NULL: return "null pointer";
    case MLPMOE_ERR_SHAPE: return "bad size";
    case MLPMOE_ERR_OFFSETS: return "bad branch offsets";
    case MLPMOE_ERR_UNSUPPORTED: return "kernel path cannot run these arguments";
    case MLPMOE_ERR_WORKSPACE: return "workspace missing, too small or misaligned";
    case MLPMOE_ERR_HIP: return "HIP runtime error";
    case MLPMOE_ERR_ALIGN: return "device pointer not 16-byte aligned";
    default: return "unknown status";
    }
}

int mlpmoe_slice(int d_inter, int B, int K_keep, const uint8_t *neuron_keep, int pad_to,
                 int32_t *branch_offsets, float *alpha, uint8_t *active_mask, int32_t *gather_index,
                 int gather_capacity)
{
    return mlpmoe_slice_rows(d_inter, B, K_keep, neuron_keep, pad_to, 1, branch_offsets, alpha, active_mask,
                             gather_index, gather_capacity);
}

int mlpmoe_slice_rows(int d_inter, int B, int K_keep, const uint8_t *neuron_keep, int pad_to, int pad_rows_to,
                      int32_t *branch_offsets, float *alpha, uint8_t *active_mask, int32_t *gather_index,
                      int gather_capacity)
{
    if (!branch_offsets || !alpha || !active_mask) return MLPMOE_ERR_NULL;
    if (B < 1 || B > MLPMOE_MAX_BRANCHES || d_inter < 0 || d_inter > (1 << 24) || pad_to < 1 ||
        pad_to > 4096 || pad_rows_to < 1 || pad_rows_to > 4096 || K_keep < 0)
        return MLPMOE_ERR_SHAPE;
    if (gather_index && gather_capacity < 0) return MLPMOE_ERR_SHAPE;

    // Sec. 3.3: keep the first K branches, rescale them by sqrt(B/K); the others are switched off.
    const bool prune = K_keep > 0 && K_keep < B;
    const float keep_alpha = prune ? (float)sqrt((double)B / (double)K_keep) : 1.0f;
    for (int b = 0; b < B; ++b) {
        const bool on = !prune || b < K_keep;
        alpha[b] = on ? keep_alpha : 0.0f;
        active_mask[b] = on ? 1 : 0;
    }

    // Sec. 3.1: contiguous slices; survivors of each slice are packed in order, then padded.
    const int base = d_inter / B, rem = d_inter % B;
    int src = 0, dst = 0;
    branch_offsets[0] = 0;
    for (int b = 0; b < B; ++b) {
        const int width = base + (b < rem ? 1 : 0);
        int kept = 0;
        for (int j = src; j < src + width; ++j) {
            if (neuron_keep && !neuron_keep[j]) continue;
            if (gather_index) {
                if (dst + kept >= gather_capacity) return MLPMOE_ERR_SHAPE;
                gather_index[dst + kept] = j;
            }
            ++kept;
        }
        const int padded = (kept + pad_to - 1) / pad_to * pad_to;
        if (gather_index) {
            if (dst + padded > gather_capacity) return MLPMOE_ERR_SHAPE;
            for (int r = kept; r < padded; ++r) gather_index[dst + r] = -1;
        }
        src += width;
        dst += padded;
        branch_offsets[b + 1] = dst;
    }
    // the compacted layer's row count (the leading dimension of its W_down) rounded up: more padding rows at
    // the end of the last branch
    const int total = (dst + pad_rows_to - 1) / pad_rows_to * pad_rows_to;
    if (gather_index) {
        if (total > gather_capacity) return MLPMOE_ERR_SHAPE;
        for (int r = dst; r < total; ++r) gather_index[r] = -1;
    }
    branch_offsets[B] = total;
    return MLPMOE_OK;
}

int mlpmoe_fade(void *W_gate, void *W_up, const int32_t *branch_offsets, const double *sparsity, int d_model,
                int d_inter, int B, int elem_bytes, float *thresholds, long long *kept, void *stream)
{
    if (B < 1 || B > MLPMOE_MAX_BRANCHES || d_model < 1 || d_inter < 0) return MLPMOE_ERR_SHAPE;
    if (!branch_offsets) return MLPMOE_ERR_NULL;
    if (branch_offsets[0] != 0 || branch_offsets[B] != d_inter) return MLPMOE_ERR_OFFSETS;
    for (int b = 0; b < B; ++b)
        if (branch_offsets[b + 1] < branch_offsets[b]) return MLPMOE_ERR_OFFSETS;
    double sched[MLPMOE_MAX_BRANCHES];
    for (int b = 0; b < B; ++b) {
        sched[b] = sparsity ? sparsity[b] : 0.9 * (double)b / (double)B;
        if (!(sched[b] >= 0.0 && sched[b] <= 1.0)) return MLPMOE_ERR_SHAPE;
    }
    for (int b = 0; b < B; ++b) {
        if (thresholds) thresholds[2 * b] = thresholds[2 * b + 1] = NAN;
        if (kept) kept[2 * b] = kept[2 * b + 1] = (long long)(branch_offsets[b + 1] - branch_offsets[b]) * d_model;
    }
    if (d_inter == 0) return MLPMOE_OK;
    if (!W_gate || !W_up) return MLPMOE_ERR_NULL;
    // 16-byte pieces: 8 bf16 values or 4 floats per row piece
    if ((elem_bytes != 2 && elem_bytes != 4) || d_model % (16 / elem_bytes) != 0) return MLPMOE_ERR_UNSUPPORTED;
    if (!aligned16(W_gate) || !aligned16(W_up)) return MLPMOE_ERR_ALIGN;

    (void)hipGetLastError();
    g_err_detail[0] = 0;
    uint32_t *scratch = nullptr;
    const size_t scratch_words = elem_bytes == 2 ? fade_scratch_words(B) : fade_scratch_words_f32(B);
    hipError_t e = hipMalloc(reinterpret_cast<void **>(&scratch), scratch_words * sizeof(uint32_t));
    if (e != hipSuccess) {
        (void)note_hip_error("hipMalloc(fade scratch)", e);
        (void)hipGetLastError();
        return MLPMOE_ERR_HIP;
    }
    int rc = MLPMOE_OK;
    void *mats[2] = {W_gate, W_up};
    for (int m = 0; m < 2 && rc == MLPMOE_OK; ++m) {
        int job[MLPMOE_MAX_BRANCHES];
        if (elem_bytes == 4) {
            double thr[MLPMOE_MAX_BRANCHES];
            long long cnt[MLPMOE_MAX_BRANCHES];
            e = launch_fade_f32(mats[m], branch_offsets, sched, B, d_model, scratch, thr, cnt, job,
                                static_cast<hipStream_t>(stream));
            if (e != hipSuccess) {
                rc = MLPMOE_ERR_HIP;
                break;
            }
            for (int b = 0; b < B; ++b) {
                if (job[b] < 0) continue;
                if (thresholds) thresholds[2 * b + m] = (float)thr[job[b]];
                if (kept) kept[2 * b + m] = cnt[job[b]];
            }
            continue;
        }
        uint32_t res[4 * MLPMOE_MAX_BRANCHES];
        e = launch_fade_bf16(mats[m], branch_offsets, sched, B, d_model, scratch, res, job,
                             static_cast<hipStream_t>(stream));
        if (e != hipSuccess) {
            rc = MLPMOE_ERR_HIP;
            break;
        }
        for (int b = 0; b < B; ++b) {
            const int j = job[b];
            if (j < 0) continue;
            const long long n = (long long)(branch_offsets[b + 1] - branch_offsets[b]) * d_model;
            const double p = sched[b] * (double)(n - 1);
            const double frac = p - (double)(long long)p;
            const uint32_t lo_bits = res[4 * j] << 16, hi_bits = res[4 * j + 1] << 16;
            float lo, hi;
            memcpy(&lo, &lo_bits, 4);
            memcpy(&hi, &hi_bits, 4);
            if (thresholds) thresholds[2 * b + m] = (float)((double)lo + frac * ((double)hi - (double)lo));
            if (kept) kept[2 * b + m] = (long long)(((unsigned long long)res[4 * j + 3] << 32) | res[4 * j + 2]);
        }
    }
    (void)hipFree(scratch);
    return rc;
}

int mlpmoe_fade_neurons(const void *W_gate, const void *W_up, const int32_t *branch_offsets,
                        const int32_t *keep_count, int d_model, int d_inter, int B, int elem_bytes,
                        uint8_t *neuron_keep, double *scores, void *stream)
{
    if (B < 1 || B > MLPMOE_MAX_BRANCHES || d_model < 1 || d_inter < 0) return MLPMOE_ERR_SHAPE;
    if (!branch_offsets || !keep_count) return MLPMOE_ERR_NULL;
    if (branch_offsets[0] != 0 || branch_offsets[B] != d_inter) return MLPMOE_ERR_OFFSETS;
    for (int b = 0; b < B; ++b) {
        if (branch_offsets[b + 1] < branch_offsets[b]) return MLPMOE_ERR_OFFSETS;
        if (keep_count[b] < 0 || keep_count[b] > branch_offsets[b + 1] - branch_offsets[b]) return MLPMOE_ERR_SHAPE;
    }
    if (d_inter == 0) return MLPMOE_OK;
    if (!W_gate || !W_up || !neuron_keep) return MLPMOE_ERR_NULL;
    if ((elem_bytes != 2 && elem_bytes != 4) || d_model % (16 / elem_bytes) != 0) return MLPMOE_ERR_UNSUPPORTED;
    if (!aligned16(W_gate) || !aligned16(W_up)) return MLPMOE_ERR_ALIGN;

    (void)hipGetLastError();
    g_err_detail[0] = 0;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const size_t score_bytes = align_up((size_t)d_inter * sizeof(double), 256);
    char *scratch = nullptr;
    hipError_t e = hipMalloc(reinterpret_cast<void **>(&scratch), score_bytes + (size_t)d_inter);
    if (e != hipSuccess) {
        (void)note_hip_error("hipMalloc(neuron scores)", e);
        (void)hipGetLastError();
        return MLPMOE_ERR_HIP;
    }
    double *d_scores = reinterpret_cast<double *>(scratch);
    uint8_t *d_keep = reinterpret_cast<uint8_t *>(scratch + score_bytes);
    e = launch_fade_neurons(W_gate, W_up, branch_offsets, keep_count, B, d_model, d_inter, elem_bytes, d_scores, d_keep, s);
    if (e == hipSuccess) {
        e = hipMemcpyAsync(neuron_keep, d_keep, (size_t)d_inter, hipMemcpyDeviceToHost, s);
        if (e == hipSuccess && scores)
            e = hipMemcpyAsync(scores, d_scores, (size_t)d_inter * sizeof(double), hipMemcpyDeviceToHost, s);
        if (e == hipSuccess) e = hipStreamSynchronize(s);
        if (e != hipSuccess) (void)note_hip_error("copying the neuron flags back", e);
    }
    (void)hipFree(scratch);
    return e == hipSuccess ? MLPMOE_OK : MLPMOE_ERR_HIP;
}

int mlpmoe_compact(const void *W_gate, const void *W_up, const void *W_down, const int32_t *gather,
                   int n_rows, int d_model, int d_inter_src, int elem_bytes, void *W_gate_c,
                   void *W_up_c, void *W_down_c, void *stream)
{
    if (n_rows < 0 || d_model < 1 || d_inter_src < 0 || (elem_bytes != 2 && elem_bytes != 4))
        return MLPMOE_ERR_SHAPE;
    if (n_rows == 0) return MLPMOE_OK;
    if (!W_gate || !W_up || !W_down || !gather || !W_gate_c || !W_up_c || !W_down_c)
        return MLPMOE_ERR_NULL;
    (void)hipGetLastError();
    hipError_t e = launch_compact(W_gate, W_up, W_down, gather, n_rows, d_model, d_inter_src,
                                  elem_bytes, W_gate_c, W_up_c, W_down_c,
                                  static_cast<hipStream_t>(stream));
    return e == hipSuccess ? MLPMOE_OK : MLPMOE_ERR_HIP;
}

size_t mlpmoe_workspace_bytes(int T, int d_model, int d_inter, int B, int elem_bytes)
{
    if (T < 0 || d_model < 1 || d_inter < 0 || B < 1 || B > MLPMOE_MAX_BRANCHES ||
        (elem_bytes != 2 && elem_bytes != 4))
        return 0;
    if (T == 0) return 256;
    size_t bytes = h_bytes(T, d_inter, elem_bytes);
    if (elem_bytes == 2) bytes += mfma_partial_bytes(T, d_model, d_inter);
    return bytes + 256 + route_scratch_bytes(T, d_inter);     // slack, then the routed path's tile tables
}

int mlpmoe_set_workspace(void *dev_ptr, size_t bytes)
{
    if (dev_ptr && ((reinterpret_cast<uintptr_t>(dev_ptr) & 255u) || bytes == 0)) return MLPMOE_ERR_WORKSPACE;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) {
        (void)note_hip_error("hipGetDevice", e);
        return MLPMOE_ERR_HIP;
    }
    std::lock_guard<std::mutex> lock(g_ws_mutex);
    DeviceWorkspace &w = g_ws[dev];
    w.user_ptr = dev_ptr;
    w.user_bytes = dev_ptr ? bytes : 0;
    return MLPMOE_OK;
}

int mlpmoe_hidden_ld(int d_inter) { return d_inter < 0 ? 0 : h_ld(d_inter); }

int mlpmoe_forward_bf16_noalloc(const void *x, const void *W_gate, const void *W_up, const void *W_down,
                                const int32_t *branch_offsets, const float *alpha, const uint8_t *active_mask,
                                int T, int d_model, int d_inter, int B, float *out, void *stream)
{
    int rc = validate_common(x, W_gate, W_up, W_down, branch_offsets, alpha, active_mask, T, d_model, d_inter, B, out);
    if (rc != MLPMOE_OK) return rc;
    if (T == 0) return MLPMOE_OK;
    const size_t need = mlpmoe_workspace_bytes(T, d_model, d_inter, B, 2);
    if (need == 0 || need > (size_t)MLPMOE_NOALLOC_SCRATCH_BYTES) {
        snprintf(g_err_detail, sizeof(g_err_detail), "mlpmoe_forward_bf16_noalloc: needs %zu bytes of scratch, has %zu",
                 need, (size_t)MLPMOE_NOALLOC_SCRATCH_BYTES);
        return MLPMOE_ERR_WORKSPACE;
    }
    void *scratch = nullptr;
    rc = noalloc_scratch(&scratch);
    if (rc != MLPMOE_OK) return rc;
    return forward_impl(x, W_gate, W_up, W_down, branch_offsets, alpha, active_mask, T, d_model, d_inter, B, out,
                        scratch, (size_t)MLPMOE_NOALLOC_SCRATCH_BYTES, MLPMOE_PATH_AUTO, true,
                        static_cast<hipStream_t>(stream));
}

int mlpmoe_forward_bf16_ws(const void *x, const void *W_gate, const void *W_up, const void *W_down,
                           const int32_t *branch_offsets, const float *alpha,
                           const uint8_t *active_mask, int T, int d_model, int d_inter, int B,
                           float *out, void *workspace, size_t workspace_bytes, int path, void *stream)
{
    return forward_impl(x, W_gate, W_up, W_down, branch_offsets, alpha, active_mask, T, d_model,
                        d_inter, B, out, workspace, workspace_bytes, path, true,
                        static_cast<hipStream_t>(stream));
}

int mlpmoe_forward_f32_ws(const float *x, const float *W_gate, const float *W_up, const float *W_down,
                          const int32_t *branch_offsets, const float *alpha,
                          const uint8_t *active_mask, int T, int d_model, int d_inter, int B,
                          float *out, void *workspace, size_t workspace_bytes, void *stream)
{
    return forward_impl(x, W_gate, W_up, W_down, branch_offsets, alpha, active_mask, T, d_model,
                        d_inter, B, out, workspace, workspace_bytes, MLPMOE_PATH_AUTO, false,
                        static_cast<hipStream_t>(stream));
}

int mlpmoe_forward_bf16(const void *x, const void *W_gate, const void *W_up, const void *W_down,
                        const int32_t *branch_offsets, const float *alpha,
                        const uint8_t *active_mask, int T, int d_model, int d_inter, int B, float *out,
                        void *stream)
{
    return forward_owned(x, W_gate, W_up, W_down, branch_offsets, alpha, active_mask, T, d_model,
                         d_inter, B, out, true, static_cast<hipStream_t>(stream));
}

int mlpmoe_forward_bf16_out_bf16(const void *x, const void *W_gate, const void *W_up, const void *W_down,
                                 const int32_t *branch_offsets, const float *alpha, const uint8_t *active_mask,
                                 int T, int d_model, int d_inter, int B, void *out, void *stream)
{
    return forward_owned(x, W_gate, W_up, W_down, branch_offsets, alpha, active_mask, T, d_model, d_inter, B,
                         static_cast<float *>(out), true, static_cast<hipStream_t>(stream), true);
}

int mlpmoe_forward_bf16_out_bf16_ws(const void *x, const void *W_gate, const void *W_up, const void *W_down,
                                    const int32_t *branch_offsets, const float *alpha,
                                    const uint8_t *active_mask, int T, int d_model, int d_inter, int B, void *out,
                                    void *workspace, size_t workspace_bytes, int path, void *stream)
{
    return forward_impl(x, W_gate, W_up, W_down, branch_offsets, alpha, active_mask, T, d_model, d_inter, B,
                        static_cast<float *>(out), workspace, workspace_bytes, path, true,
                        static_cast<hipStream_t>(stream), true);
}

int mlpmoe_forward(const void *x, const void *W_gate, const void *W_up, const void *W_down,
                   const int32_t *branch_offsets, const float *alpha, const uint8_t *active_mask, int T,
                   int d_model, int d_inter, int B, float *out, void *stream)
{
    return mlpmoe_forward_bf16(x, W_gate, W_up, W_down, branch_offsets, alpha, active_mask, T,
                               d_model, d_inter, B, out, stream);
}

int mlpmoe_forward_f32(const float *x, const float *W_gate, const float *W_up, const float *W_down,
                       const int32_t *branch_offsets, const float *alpha, const uint8_t *active_mask,
                       int T, int d_model, int d_inter, int B, float *out, void *stream)
{
    return forward_owned(x, W_gate, W_up, W_down, branch_offsets, alpha, active_mask, T, d_model,
                         d_inter, B, out, false, static_cast<hipStream_t>(stream));
}

static int forward_routed(const void *x, const void *Wg, const void *Wu, const void *Wd, const int32_t *off,
                          const float *alpha, const uint8_t *mask, const uint8_t *route, int T, int d_model,
                          int d_inter, int B, float *out, void *workspace, size_t workspace_bytes, bool own,
                          hipStream_t stream, bool is_bf16 = true)
{
    int rc = validate_common(x, Wg, Wu, Wd, off, alpha, mask, T, d_model, d_inter, B, out);
    if (rc != MLPMOE_OK) return rc;
    if (T == 0) return MLPMOE_OK;
    if (!route) return MLPMOE_ERR_NULL;
    std::unique_lock<std::mutex> lock(g_ws_mutex, std::defer_lock);
    if (own) {
        lock.lock();                                   // held until the kernels are enqueued
        rc = owned_workspace(mlpmoe_workspace_bytes(T, d_model, d_inter, B, is_bf16 ? 2 : 4), stream, &workspace,
                             &workspace_bytes);
        if (rc != MLPMOE_OK) return rc;
    }
    BranchTable bt;
    build_table(off, alpha, mask, B, bt);
    return forward_table(bt, is_bf16 && fast_path_aligned(bt, d_model, d_inter), x, Wg, Wu, Wd, T, d_model, d_inter,
                         out, workspace, workspace_bytes, MLPMOE_PATH_AUTO, is_bf16, stream, route);
}

int mlpmoe_forward_routed_f32(const float *x, const float *W_gate, const float *W_up, const float *W_down,
                              const int32_t *branch_offsets, const float *alpha, const uint8_t *active_mask,
                              const uint8_t *route, int T, int d_model, int d_inter, int B, float *out, void *stream)
{
    return forward_routed(x, W_gate, W_up, W_down, branch_offsets, alpha, active_mask, route, T, d_model, d_inter,
                          B, out, nullptr, 0, true, static_cast<hipStream_t>(stream), false);
}

int mlpmoe_forward_routed_f32_ws(const float *x, const float *W_gate, const float *W_up, const float *W_down,
                                 const int32_t *branch_offsets, const float *alpha, const uint8_t *active_mask,
                                 const uint8_t *route, int T, int d_model, int d_inter, int B, float *out,
                                 void *workspace, size_t workspace_bytes, void *stream)
{
    return forward_routed(x, W_gate, W_up, W_down, branch_offsets, alpha, active_mask, route, T, d_model, d_inter,
                          B, out, workspace, workspace_bytes, false, static_cast<hipStream_t>(stream), false);
}

int mlpmoe_forward_routed_bf16(const void *x, const void *W_gate, const void *W_up, const void *W_down,
                               const int32_t *branch_offsets, const float *alpha, const uint8_t *active_mask,
                               const uint8_t *route, int T, int d_model, int d_inter, int B, float *out,
                               void *stream)
{
    return forward_routed(x, W_gate, W_up, W_down, branch_offsets, alpha, active_mask, route, T, d_model, d_inter,
                          B, out, nullptr, 0, true, static_cast<hipStream_t>(stream));
}

int mlpmoe_forward_routed_bf16_ws(const void *x, const void *W_gate, const void *W_up, const void *W_down,
                                  const int32_t *branch_offsets, const float *alpha,
                                  const uint8_t *active_mask, const uint8_t *route, int T, int d_model,
                                  int d_inter, int B, float *out, void *workspace, size_t workspace_bytes,
                                  void *stream)
{
    return forward_routed(x, W_gate, W_up, W_down, branch_offsets, alpha, active_mask, route, T, d_model, d_inter,
                          B, out, workspace, workspace_bytes, false, static_cast<hipStream_t>(stream));
}

struct mlpmoe_plan {
    BranchTable bt;
    int d_model, d_inter, B, elem_bytes, max_T, device;
    bool aligned;
    void *ws;
    size_t ws_bytes;
};

int mlpmoe_plan_create(const int32_t *branch_offsets, const float *alpha, const uint8_t *active_mask,
                       int d_model, int d_inter, int B, int elem_bytes, int max_T, mlpmoe_plan **plan)
{
    if (!plan) return MLPMOE_ERR_NULL;
    *plan = nullptr;
    if ((elem_bytes != 2 && elem_bytes != 4) || max_T < 1) return MLPMOE_ERR_SHAPE;
    // same table checks as a forward call, with stand-in data pointers (T = 0 skips those)
    int rc = validate_common(nullptr, nullptr, nullptr, nullptr, branch_offsets, alpha, active_mask, 0, d_model,
                             d_inter, B, nullptr);
    if (rc != MLPMOE_OK) return rc;
    mlpmoe_plan *p = new (std::nothrow) mlpmoe_plan();
    if (!p) return MLPMOE_ERR_WORKSPACE;
    build_table(branch_offsets, alpha, active_mask, B, p->bt);
    p->d_model = d_model;
    p->d_inter = d_inter;
    p->B = B;
    p->elem_bytes = elem_bytes;
    p->max_T = max_T;
    p->aligned = elem_bytes == 2 && fast_path_aligned(p->bt, d_model, d_inter);
    // Workspace for every T up to max_T.  H grows with T; the split-K partials are T times a
    // split factor that is constant while T stays inside one row of token tiles (64, 128 or 256 tokens),
    // so the maximum over a tile row is at its last T: checking the multiples of 64 and max_T covers all.
    p->ws_bytes = 0;
    for (long long t = 64; ; t += 64) {
        const int tt = t < max_T ? (int)t : max_T;
        p->ws_bytes = std::max(p->ws_bytes, mlpmoe_workspace_bytes(tt, d_model, d_inter, B, elem_bytes));
        if (tt == max_T) break;
    }
    p->ws = nullptr;
    (void)hipGetLastError();
    g_err_detail[0] = 0;
    hipError_t e = hipGetDevice(&p->device);
    if (e == hipSuccess && p->ws_bytes) e = hipMalloc(&p->ws, p->ws_bytes);
    if (e != hipSuccess) {
        (void)note_hip_error("mlpmoe_plan_create: device workspace", e);
        (void)hipGetLastError();
        delete p;
        return MLPMOE_ERR_HIP;
    }
    *plan = p;
    return MLPMOE_OK;
}

int mlpmoe_plan_forward(const mlpmoe_plan *plan, const void *x, const void *W_gate, const void *W_up,
                        const void *W_down, int T, float *out, void *stream)
{
    if (!plan) return MLPMOE_ERR_NULL;
    if (T < 0 || T > plan->max_T) return MLPMOE_ERR_SHAPE;
    if (T == 0) return MLPMOE_OK;
    if (!x || !out || (plan->d_inter > 0 && (!W_gate || !W_up || !W_down))) return MLPMOE_ERR_NULL;
    if (!aligned16(x) || !aligned16(out) || !aligned16(W_gate) || !aligned16(W_up) || !aligned16(W_down))
        return MLPMOE_ERR_ALIGN;
    return forward_table(plan->bt, plan->aligned, x, W_gate, W_up, W_down, T, plan->d_model, plan->d_inter, out,
                         plan->ws, plan->ws_bytes, MLPMOE_PATH_AUTO, plan->elem_bytes == 2,
                         static_cast<hipStream_t>(stream));
}

int mlpmoe_plan_destroy(mlpmoe_plan *plan)
{
    if (!plan) return MLPMOE_OK;
    int rc = MLPMOE_OK;
    if (plan->ws) {
        int cur = 0;
        (void)hipGetDevice(&cur);
        if (hipSetDevice(plan->device) != hipSuccess || hipDeviceSynchronize() != hipSuccess ||
            hipFree(plan->ws) != hipSuccess)
            rc = MLPMOE_ERR_HIP;
        (void)hipSetDevice(cur);
    }
    delete plan;
    return rc;
}

int mlpmoe_release(void)
{
    std::lock_guard<std::mutex> lock(g_ws_mutex);
    int rc = MLPMOE_OK;
    int cur = 0;
    (void)hipGetDevice(&cur);
    for (auto &kv : g_ws) {
        if (!kv.second.ptr) continue;
        if (hipSetDevice(kv.first) != hipSuccess || hipDeviceSynchronize() != hipSuccess ||
            hipFree(kv.second.ptr) != hipSuccess)
            rc = MLPMOE_ERR_HIP;
        kv.second = DeviceWorkspace();
    }
    (void)hipSetDevice(cur);
    return rc;
}

}  // extern "C"
