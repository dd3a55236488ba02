// Internal state of a libngc context.  Host side only; no kernel includes this
// for anything but the table layouts below.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>
#include <memory>
#include <string>
#include <vector>

#include "../../include/ngc.h"
#include "ngc_host_pool.h"

constexpr int NGC_MAX_N = 64;
constexpr int NGC_MAX_PROFILE = 4096;

// One layer's encoding matrix in compressed-row form: the non-zeros of row i are
// entries rowptr[i] .. rowptr[i+1]-1 of (col, coef).
struct ngc_layer_code {
    bool set = false;
    // explicit decoding matrix A_sigma (Def. 1), one row per straggler set of size sigma in
    // lexicographic order; empty until ngc_build_decoding_table
    std::vector<double> A;
    int64_t A_rows = 0;
    double* d_A = nullptr;  // device copy, uploaded on first use
    bool A_stale = true;    // host table changed since the upload
    std::vector<double> B;      // n x k dense, fp64, as given
    std::vector<int> rowptr;    // n + 1
    std::vector<int> col;
    std::vector<double> coef;
    std::vector<double> row_norm;  // ||b_i||_2, n entries (guarded layer choice)
    // full-response factor for decode-vector selection (ngc_solve.cpp): least-norm a0 with
    // a0^T B = 1^T and an orthonormal basis N (n x q, row-major) of {v : v^T B = 0};
    // null_ok is false when B has no exact full-response solution
    std::vector<double> a0, N;
    int q = 0;
    bool null_ok = false;
};

struct ngc_profile_rec {
    int kernel;
    hipEvent_t start, stop;
};

struct ngc_ctx {
    int n = 0;   // workers
    int k = 0;   // partitions, k = c * n
    int c = 1;   // partitions per atomic task (Sec. II-C)
    int L = 0;
    int64_t d = 0;
    std::vector<int> s;
    hipStream_t stream = nullptr;
    std::vector<ngc_layer_code> code;
    double guard_limit = 0.0;  // guarded layer choice: limit on kappa_hat, 0 = off (ngc_set_decode_guard)

    // MLP shape (NGC_LOSS_MLP2)
    int mlp_din = 0, mlp_hidden = 0, mlp_classes = 0;

    // device-side private state, created on first use
    bool dev_ready = false;
    int cu_count = 0;
    bool code_dirty = true;          // host tables changed since the last upload
    void* d_code = nullptr;          // packed tables for all layers (see ngc_device.hip)
    size_t d_code_bytes = 0;
    size_t code_nnz = 0;             // non-zeros over all layers in d_code
    size_t code_gmask_off = 0;       // byte offsets of the worker-group tables inside d_code
    size_t code_gcoef_off = 0;
    int code_ng = 0, code_kp = 0;    // groups of four workers, k rounded up to a multiple of 4
    int lds_limit = 0;               // LDS bytes one block may use on this device
    // per-round records of ngc_coded_rounds: device table, pinned staging, event after the copy
    void* d_rounds = nullptr;
    void* h_rounds = nullptr;
    size_t rounds_cap = 0;           // records both hold
    hipEvent_t rounds_ev = nullptr;
    bool rounds_ev_set = false;
    // the records travel on a stream of the library's own (default priority), so that a run's
    // copy overlaps the kernel of the run before it; one event per run orders kernel after copy
    hipStream_t rounds_copy_stream = nullptr;
    std::vector<hipEvent_t> rounds_run_ev;
    std::unique_ptr<ngc_host_pool> pool;  // host threads for the bookkeeping of many rounds, created on first need
    float* d_ws = nullptr;           // workspace: block partials / residuals / MLP activations
    size_t d_ws_bytes = 0;
    // worker mode: unit -> partition / output-row maps, two copies used in turn so that a call
    // can fill one while the kernels of the previous call still read the other
    int* d_maps[2] = {nullptr, nullptr};
    int* h_maps[2] = {nullptr, nullptr};  // pinned staging
    size_t maps_cap = 0;                  // ints per copy
    hipEvent_t maps_ev[2] = {nullptr, nullptr};
    bool maps_ev_set[2] = {false, false};
    int maps_turn = 0;
    int* d_wtab = nullptr;                // worker-encode tables, rebuilt when a code changes
    size_t d_wtab_bytes = 0;
    bool wtab_dirty = true;
    int wtab_T = 0;

    unsigned profile_mask = 0;       // bit k: time launches of kernel id k
    bool prof_suspended = false;     // set while an entry point that must not create events runs
    std::vector<ngc_profile_rec> prof;
    std::vector<hipEvent_t> event_pool;

    mutable std::string err;
};

int ngc_fail(const ngc_ctx* ctx, int code, const std::string& msg);
// Status for a C++ exception caught at the C boundary (called inside a catch block): no
// exception leaves the library.
int ngc_on_exception();

// defined in ngc_device.hip
void ngc_dev_release(ngc_ctx* ctx);

// Layered task schedule of every worker derived from the code tables (ngc_host.cpp):
// order[i] = partitions in the order worker i computes them (c per atomic task),
// needed[u*n+i] = atomic tasks worker i must have finished to form its layer-u message,
// T = longest schedule in atomic tasks.  All layers must be set.
struct ngc_worker_plan {
    std::vector<std::vector<int>> order;
    std::vector<int> needed;
    int T = 0;
};
int ngc_make_worker_plan(const ngc_ctx* ctx, ngc_worker_plan& plan);

// defined in ngc_solve.cpp: least-norm a_S with a_S^T B_S = 1^T.
// rows: indices of responders (size ns).  B: n x k row-major.  a_out: n entries,
// zero outside rows.  Returns the numerical rank found; resid = max_j |a^T B - 1|.
int ngc_min_norm_decode(const double* B, int n, int k, const int* rows, int ns, double* a_out,
                        double* resid);
// Full-response factor of B (n x k): a0 [n], N [n][q] row-major; returns q = n - rank(B).
// resid = max_j |a0^T B - 1|.
int ngc_null_factor(const double* B, int n, int k, double* a0, double* N, double* resid);
// The same vector as ngc_min_norm_decode, obtained from the factor: one small system with an
// equation per straggler.  rows ascending.
int ngc_min_norm_decode_null(const double* B, int n, int k, const double* a0, const double* N,
                             int q, const int* rows, int ns, double* a_out, double* resid);
// Layer choice and decode vector for one straggler mask (the work of ngc_select_decode_vec)
// without touching the context's error text, so that several host threads may call it at once.
int ngc_select_core(const ngc_ctx* ctx, const uint8_t* mask, int* layer_out, double* a_out,
                    double* residual_out, bool first_only);
// Decode vector of layer `layer` for the responders in rows (ascending), by whichever of the
// two routes is cheaper for this code and straggler count.
void ngc_layer_decode_vec(const ngc_ctx* ctx, int layer, const int* rows, int ns, double* a_out,
                          double* resid);
