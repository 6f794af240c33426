// Internal declarations shared by the translation units of libsom (not part of the public ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <utility>
#include <vector>

#include "som.h"

namespace som {

constexpr int kNodesPerStage = 128;   // nodes of W staged through LDS at a time by the BMU kernel
constexpr int kMaxStepsResident = 32; // BMU kernel keeps a sample's features in registers up to D = 64

struct BmuPrep {
    float* stage = nullptr;        // [Kpad / 128][nch] blobs: 128 padded weight rows of a chunk, then -|w|^2 / 2
    void* stage16 = nullptr;       // bf16 hi/lo stage rows of the split search (4 <= D <= 64), else null
    float* wwin = nullptr;         // [Kpad][kb][2][8] the same slots as stage16 in float32 (centred, zeros off-window)
    int kb = 0;                    // whole 16-feature blocks of a stage16 row
    int tail_r = 0;                // features of the packed tail block behind them (0: none; D <= 64 only)
    int nch16 = 0;                 // chunks of a stage in stage16 (1 for D <= 64, 64-feature chunks above)
    float* wt = nullptr;           // [D][Kpad] transposed weights (as given, not centred)
    float* centre = nullptr;       // [D] column means of W; stage rows and sample registers hold values minus this
    // [0] = bits of max_k |w_k - centre|^2, [1], [2] = recheck-list length (alternating calls), [3] = total,
    // [4], [5] = length of the second list (samples whose candidate slots overflowed; alternating calls)
    unsigned int* scal = nullptr;
    int kpad = 0, steps = 0, stride = 0;
    int nch = 1;                   // feature chunks of 2 * steps features (1 unless D > 64)
    int calls = 0;                 // bmu_run calls served by this preparation (selects the list counter)
};

struct BmuArgs {
    const float* X;
    int64_t ldx;
    const uint32_t* idx;
    int64_t m;
    int32_t D, K, kpad;
    const float* W;          // caller's dense K x D weights (exact distances)
    const float* stage;      // BmuPrep::stage
    int32_t stride;          // BmuPrep::stride (floats per row of the float32 stage)
    const void* stage16;     // BmuPrep::stage16 (null: float32 search)
    const float* wwin;       // BmuPrep::wwin
    int32_t tail_r;          // BmuPrep::tail_r
    void* parts;             // split search, D > 64: the pass's samples as bf16 parts, [m][chunks * 8][hi x 8 | lo x 8]
    const float* wt;         // BmuPrep::wt
    const float* centre;     // BmuPrep::centre
    unsigned int* scal;      // BmuPrep::scal
    int32_t slot;            // which of scal[1], scal[2] this call counts into
    int64_t full_tiles;      // bmu_kernel: workgroups below this number take full tiles, the others half tiles
    float* cut_all;          // [m] per presented sample: its cut when it is to be re-decided, a NaN otherwise
    uint32_t* recheck;       // [m] sample positions to re-decide (compacted from cut_all by bmu_list_kernel)
    // Candidate pass (long lists only): the search is repeated for the listed samples, and every node whose score
    // reaches the sample's cut is noted; direct differences are then taken over those few nodes only.
    float* cutv;             // [m] per list entry: best score minus the rounding bound
    ulonglong2* cand;        // [cand_cap][2]: per list entry and half-wavefront, seven 16-bit node ids and their count
    uint32_t* recheck2;      // [cand_cap] samples left to the all-nodes pass (slots overflowed, or no candidate)
    int32_t slot2;           // which of scal[4], scal[5] counts recheck2
    uint32_t cand_min;       // the candidate pass serves list lengths in (cand_min, cand_cap]
    uint32_t cand_cap;
    int32_t* bmu;            // [m], always written
    float* d2;               // may be null
    double* qe;              // [2], accumulated (caller zeroes); may be null
    double* qe_part;         // [kQeSlots][2] partial sums of this call (zero on entry, zeroed again by qe_finish_kernel)
};

constexpr int kQeSlots = 256;
constexpr int kMaxDevices = 64;                 // devices the per-device tables hold
constexpr int kUpdateStaticCells = 65536;       // som_neighborhood_update_static: K * (D + 1) at most
constexpr int kUpdateStaticNodes = 32768;       // and K at most
constexpr int kCandSlots = 8;         // 16-bit places per (list entry, half-wavefront): up to seven node ids and a count

} // namespace som

struct som_ctx {
    int device = 0;
    int units = 0;                 // compute units of the device (queried on first use)
    hipStream_t stream = nullptr;
    hipStream_t copy_stream = nullptr;
    char err[512] = {0};
    double eta = 1.0, mu = 0.0;    // update rule (som_set_update_rule)
    float* velocity = nullptr;

    // BMU workspaces (grown on demand)
    void* prep_blob = nullptr;
    size_t prep_bytes = 0;
    uint32_t* recheck = nullptr;   // one allocation: sample positions [cap], cuts [cap], second list, candidate slots
    size_t recheck_cap = 0;
    int32_t* bmu_ws = nullptr;     // BMU indices of the epoch drivers (one chunk's worth)
    size_t bmu_elems = 0;
    void* acc_blob = nullptr;      // per-workgroup float64 slices + counts of the accumulation pass
    void* parts_blob = nullptr;    // the presented samples of a pass as bf16 parts (split search, D > 64)
    size_t parts_bytes = 0;
    size_t acc_bytes = 0;
    void* upd_blob = nullptr;      // influence matrix + split-k partials of the update
    size_t upd_bytes = 0;
    double* upd_static = nullptr;  // this device's fixed update workspace (som_neighborhood_update_static)
    int safeguard = 0;             // SOM_SAFEGUARD_*
    int reproducible = 0;          // prefer the fixed-order accumulation kernel
    int search = 0;                // SOM_SEARCH_*
    double* qe_part = nullptr;     // [kQeSlots][2], zero between calls
    void* topo_blob = nullptr;     // node distances, adjacency matrix and lists of the topology rebuild
    size_t topo_bytes = 0;
    // epoch-internal accumulators
    double* S = nullptr;
    size_t S_elems = 0;
    unsigned long long* n = nullptr;
    size_t n_elems = 0;
    double* qe = nullptr;          // double[2]
    int32_t* small = nullptr;      // int32[4]: n_guarded, n_empty, spare
    void* host_small = nullptr;    // pinned mirror for reading results back
    // streaming
    float* pinned[2] = {nullptr, nullptr};
    float* dchunk[2] = {nullptr, nullptr};
    size_t chunk_elems = 0;
    hipEvent_t ev_copied[2] = {nullptr, nullptr};
    hipEvent_t ev_consumed[2] = {nullptr, nullptr};
    hipEvent_t ev_t[4] = {nullptr, nullptr, nullptr, nullptr};
    std::vector<hipEvent_t> h2d_events;   // (start, stop) per chunk of a streamed epoch; grown on demand, reused
    // measurement support: event pairs around every launch of the main BMU kernel while profiling is on
    bool profiling = false;
    std::vector<std::pair<hipEvent_t, hipEvent_t>> prof_events;
    size_t prof_used = 0;
};

namespace som {

int fail(som_ctx* ctx, int code, const char* fmt, ...);
int check_hip(som_ctx* ctx, hipError_t e, const char* what);

// kernels' host launchers (each returns SOM_OK or an error code after recording detail in ctx)
int launch_fill_zero(som_ctx* ctx, void* p, size_t bytes);
// qe (double[2]) and small (int32[4]) are zeroed by the preparation kernel when given
int bmu_prepare(som_ctx* ctx, const float* W, int32_t K, int32_t D, BmuPrep* out, double* qe, int32_t* small);
int bmu_run(som_ctx* ctx, BmuPrep& prep, BmuArgs args);
int accumulate_run(som_ctx* ctx, const float* X, int32_t D, int64_t ldx, const uint32_t* idx, int64_t m,
                   const int32_t* bmu, int32_t K, double* S, unsigned long long* n, bool zero_first);
// 1 = shape not served by the MFMA path (caller falls back), otherwise SOM_OK or an error code
int accumulate_mfma_run(som_ctx* ctx, const float* X, int32_t D, int64_t ldx, const uint32_t* idx, int64_t m,
                        const int32_t* bmu, int32_t K, double* S, unsigned long long* n, bool zero_first);
int accumulate_f64_run(som_ctx* ctx, const float* X, int32_t D, int64_t ldx, const uint32_t* idx, int64_t m,
                        const int32_t* bmu, int32_t K, double* S, unsigned long long* n, bool zero_first);
int update_run(som_ctx* ctx, const double* S, const unsigned long long* n, const float* G, int32_t K,
               int32_t D, double sigma, double eps_h, float* W, int32_t* small);
int update_static_init(som_ctx* ctx);
int update_static_run(som_ctx* ctx, const double* S, const unsigned long long* n, const float* G, int32_t K,
                      int32_t D, double sigma, double eps_h, float* W, int32_t* small);

} // namespace som
