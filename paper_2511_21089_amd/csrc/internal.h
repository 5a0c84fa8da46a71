// Internal declarations shared by the host API and the kernel translation units.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "mlpmoe.h"

namespace mlpmoe {

constexpr int kMaxRuns = MLPMOE_MAX_BRANCHES / 2 + 1;

// Branch table of one call, passed to kernels by value (kernel-argument memory).
// A "run" is a maximal range of neurons covered by consecutive active, non-empty
// branches: since alpha_b is folded into the gated intermediate, the down
// projection may sweep a whole run without looking at branch boundaries.
struct BranchTable {
    int B;
    int n_runs;
    int d_eff;                               // neurons in active branches
    int off[MLPMOE_MAX_BRANCHES + 1];
    float alpha[MLPMOE_MAX_BRANCHES];
    unsigned long long active;               // bit b set: branch b is computed
    int run_start[kMaxRuns];
    int run_end[kMaxRuns];
};

struct FwdArgs {
    const void *x, *Wg, *Wu, *Wd;
    float *out;         // [T, d_model] float, or the same number of bf16 values when out_bf16
    bool out_bf16 = false;
    int T, d_model, d_inter;
    void *H;            // gated intermediate [T, ldh], bf16 or float
    int ldh;
    float *partial;     // split-K partial sums, or nullptr
    size_t partial_bytes;
    const uint8_t *route = nullptr;   // per-token routing [T, B] (device), or nullptr
    uint8_t *route_scratch = nullptr; // route_scratch_bytes(T, d_inter) bytes for the routed MFMA path (device)
    int tile_shape = -1;              // MFMA kernels: -1 = chosen from the sizes, else a TileShape (MLPMOE_PATH_MFMA_* - MLPMOE_PATH_MFMA_WIDE)
    hipStream_t stream;
};

extern thread_local char g_err_detail[192];

// Fractal Fade of one bf16 projection matrix (see kernels_fade.hip); synchronises the stream.
hipError_t launch_fade_bf16(void *W, const int32_t *off, const double *sparsity, int B, int d_model,
                            uint32_t *scratch, uint32_t *host_result, int *job_of_branch, hipStream_t s);
size_t fade_scratch_words(int B);
// The same for a float matrix; thresholds / kept are per job (job_of_branch maps branches to jobs).
hipError_t launch_fade_f32(void *W, const int32_t *off, const double *sparsity, int B, int d_model,
                           uint32_t *scratch, double *thresholds, long long *kept, int *job_of_branch, hipStream_t s);
size_t fade_scratch_words_f32(int B);
// Structured form (whole neurons): scores and keep flags of all neurons, asynchronous on s.
// elem_bytes: 2 (bf16, d_model a multiple of 8) or 4 (float, a multiple of 4).
hipError_t launch_fade_neurons(const void *Wg, const void *Wu, const int32_t *off, const int32_t *keep_count,
                               int B, int d_model, int d_inter, int elem_bytes, double *scores, uint8_t *keep,
                               hipStream_t s);

// Records which runtime call failed and how (read back through mlpmoe_last_error_detail()).
// Returns e, so that a failing site can `return note_hip_error("...", e);`.
hipError_t note_hip_error(const char *where, hipError_t e);

// Status of the launch just made; on failure notes `where` and hands the code back.
inline hipError_t launch_status(const char *where)
{
    const hipError_t e = hipGetLastError();
    return e == hipSuccess ? e : note_hip_error(where, e);
}

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

// Leading dimension of the intermediate H (elements).
inline int h_ld(int d_inter) { return (int)align_up((size_t)(d_inter > 0 ? d_inter : 1), 64); }

// Split-K factor of the MFMA down projection for an output of T x d_model and kt K-tiles.
int mfma_down_splits(int T, int d_model, int k_elems);
size_t mfma_partial_bytes(int T, int d_model, int d_inter);

hipError_t launch_fill_zero(float *out, size_t n, hipStream_t s);
hipError_t launch_fill_zero16(uint16_t *out, size_t n, hipStream_t s);
hipError_t launch_generic(const FwdArgs &a, const BranchTable &bt, bool is_bf16);
hipError_t launch_mfma_bf16(const FwdArgs &a, const BranchTable &bt);
size_t route_scratch_bytes(int T, int d_inter);
hipError_t launch_mfma_routed_bf16(const FwdArgs &a, const BranchTable &bt);
hipError_t launch_decode_bf16(const FwdArgs &a, const BranchTable &bt);
hipError_t launch_decode_routed_bf16(const FwdArgs &a, const BranchTable &bt);
hipError_t launch_compact(const void *Wg, const void *Wu, const void *Wd, const int32_t *gather,
                          int n_rows, int d_model, int d_inter_src, int elem_bytes, void *Wg_c,
                          void *Wu_c, void *Wd_c, hipStream_t s);


// Brackets one kernel launch with a pair of events when profiling is enabled.
void profile_mark(int kernel_id, hipStream_t s, bool begin);
struct ProfileScope {
    int id;
    hipStream_t s;
    ProfileScope(int kernel_id, hipStream_t stream) : id(kernel_id), s(stream) { profile_mark(id, s, true); }
    ~ProfileScope() { profile_mark(id, s, false); }
};

}  // namespace mlpmoe
