// C-ABI front end: argument validation, routing to a kernel family, status strings.
// All checks run before the first HIP call so they can be exercised without a GPU.
#include "../../include/lsm.h"
#include "../../include/lsm_bench.h"
#include "lsm_internal.h"

#include <mutex>
#include <vector>

namespace lsm {
namespace {
struct ProfRec { int id; hipEvent_t t0, t1; };
std::mutex g_prof_mu;
// Benchmark-only, process-wide state (declared in lsm_bench.h, outside the thread-safety contract of lsm.h):
// off unless lsm_profile_start() was called.
bool g_prof_on = false, g_prof_open = false;
std::vector<ProfRec> g_prof;
}  // namespace

void prof_begin(int kernel_id, hipStream_t stream) {
    if (!g_prof_on) return;
    std::lock_guard<std::mutex> lk(g_prof_mu);
    ProfRec r{kernel_id, nullptr, nullptr};
    g_prof_open = false;
    if (hipEventCreate(&r.t0) != hipSuccess) return;
    if (hipEventCreate(&r.t1) != hipSuccess) {
        (void)hipEventDestroy(r.t0);
        return;
    }
    (void)hipEventRecord(r.t0, stream);
    g_prof.push_back(r);
    g_prof_open = true;
}
void prof_end(hipStream_t stream) {
    if (!g_prof_on) return;
    std::lock_guard<std::mutex> lk(g_prof_mu);
    // only the record that the matching prof_begin opened (none if its events could not be created)
    if (g_prof_open && !g_prof.empty()) (void)hipEventRecord(g_prof.back().t1, stream);
    g_prof_open = false;
}
}  // namespace lsm

namespace {

bool dim_ok(int d) { return d == 64 || d == 128 || d == 256; }
bool chunk_ok(int c) { return c == 16 || c == 32 || c == 64 || c == 128; }
bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

int check_params(const lsm_params* p, lsm::Dims* d) {
    if (!p) return LSM_ERR_NULL;
    if (p->struct_size != sizeof(lsm_params)) return LSM_ERR_SHAPE;
    if (p->B < 1 || p->H < 1 || p->T < 1 || p->d_k < 1 || p->d_v < 1 || p->chunk_size < 1) return LSM_ERR_SHAPE;
    if (p->decay_kind < 0 || p->decay_kind > 3) return LSM_ERR_UNSUPPORTED;
    if (p->dtype != LSM_DTYPE_F32 && p->dtype != LSM_DTYPE_BF16) return LSM_ERR_UNSUPPORTED;
    if (!dim_ok(p->d_k) || !dim_ok(p->d_v) || !chunk_ok(p->chunk_size)) return LSM_ERR_UNSUPPORTED;
    // index arithmetic inside the kernels is 64-bit, grid dimensions are not
    const long long bh = (long long)p->B * p->H;
    if (p->layout != LSM_LAYOUT_BHTD && p->layout != LSM_LAYOUT_BTHD) return LSM_ERR_UNSUPPORTED;
    if (p->flags & ~(LSM_FLAG_SAVE_STATES | LSM_FLAG_SAVE_ALWAYS)) return LSM_ERR_UNSUPPORTED;
    if ((p->flags & LSM_FLAG_SAVE_ALWAYS) && !(p->flags & LSM_FLAG_SAVE_STATES)) return LSM_ERR_UNSUPPORTED;
    if (p->n_seq < 0 || (p->n_seq > 0 && p->B != 1)) return LSM_ERR_SHAPE;
    if ((p->n_seq > 0) != (p->cu_seqlens != nullptr)) return LSM_ERR_NULL;
    if (misaligned(p->cu_seqlens)) return LSM_ERR_ALIGN;
    // packed input: every sequence adds at most one ragged chunk to the count
    const long long n = ((long long)p->T + p->chunk_size - 1) / p->chunk_size + p->n_seq;
    const long long seqs = p->n_seq ? (long long)p->n_seq * p->H : bh;
    if (bh > 65535 || seqs > 65535 || n > 0x7fffffffLL || bh * p->T > (1LL << 40)) return LSM_ERR_SHAPE;
    d->B = p->B; d->H = p->H; d->T = p->T; d->dk = p->d_k; d->dv = p->d_v; d->C = p->chunk_size;
    d->N = int(n); d->kind = p->decay_kind; d->bf16 = p->dtype == LSM_DTYPE_BF16;
    d->layout = p->layout; d->nseq = p->n_seq; d->cu = p->cu_seqlens; d->cstart = nullptr;
    // Only the matrix-core kernels keep states between the two calls; elsewhere the flag changes nothing.
    // (the scalar kinds with d_v = 256 run one pass per 128-wide value slice over a shared workspace and keep nothing)
    d->save = (p->flags & LSM_FLAG_SAVE_STATES) != 0 && lsm::mfma_supported(*d) && (d->kind == 3 || d->dv == 128);
    return LSM_OK;
}

// packed input: the first bytes of the workspace hold the first chunk of every sequence
size_t table_bytes(const lsm::Dims& d) { return d.nseq ? lsm::align256(size_t(d.nseq + 1) * sizeof(int)) : 0; }
hipError_t prepare_tables(lsm::Dims& d, void*& workspace, hipStream_t stream) {
    if (!d.nseq) return hipSuccess;
    int* cstart = static_cast<int*>(workspace);
    workspace = static_cast<char*>(workspace) + table_bytes(d);
    d.cstart = cstart;
    return lsm::launch_chunk_starts(d, cstart, stream);
}

}  // namespace

// ---- scratch of the entry point that allocates nothing -------------------------------------------------
// A file-scope device array: every GPU the library runs on holds its own copy, at its own address, until
// the process ends.  Its name is a host-side stand-in; the device address comes from hipGetSymbolAddress,
// once per device, and only that pointer is ever handed to a kernel.
namespace {
constexpr size_t kScratchBytes = LSM_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

std::mutex g_scratch_mu;
void* g_scratch_ptr[64] = {};  // per device, filled on the first call on that device (a once-initialised cache)

hipError_t scratch_of_current_device(void** out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}
}  // namespace

extern "C" {

int lsm_version(void) { return 6; }

const char* lsm_status_string(int status) {
    switch (status) {
        case LSM_OK: return "ok";
        case LSM_ERR_NULL: return "a required pointer is NULL or a forbidden pointer is not NULL";
        case LSM_ERR_SHAPE: return "bad dimension or struct_size";
        case LSM_ERR_UNSUPPORTED: return "unsupported d_k/d_v/chunk_size/decay_kind/dtype";
        case LSM_ERR_ALIGN: return "pointer not 16-byte aligned";
        case LSM_ERR_WORKSPACE: return "workspace missing or too small (or, without a workspace argument, larger than the built-in scratch)";
        case LSM_ERR_LAUNCH: return "HIP error while enqueuing kernels";
        default: return "unknown status";
    }
}

int lsm_profile_start(void) {
    std::lock_guard<std::mutex> lk(lsm::g_prof_mu);
    for (auto& r : lsm::g_prof) { (void)hipEventDestroy(r.t0); (void)hipEventDestroy(r.t1); }
    lsm::g_prof.clear();
    lsm::g_prof_on = true;
    return LSM_OK;
}

int lsm_profile_stop(int* kernel_ids, float* milliseconds, int capacity) {
    std::lock_guard<std::mutex> lk(lsm::g_prof_mu);
    lsm::g_prof_on = false;
    int n = 0;
    for (auto& r : lsm::g_prof) {
        float ms = 0.f;
        if (hipEventSynchronize(r.t1) == hipSuccess && hipEventElapsedTime(&ms, r.t0, r.t1) == hipSuccess &&
            n < capacity && kernel_ids && milliseconds) {
            kernel_ids[n] = r.id;
            milliseconds[n] = ms;
            ++n;
        }
        (void)hipEventDestroy(r.t0);
        (void)hipEventDestroy(r.t1);
    }
    lsm::g_prof.clear();
    return n;
}

const char* lsm_kernel_name(int kernel_id) {
    static const char* names[lsm::KID_COUNT] = {
        "generic_cumsum", "generic_chunk_state", "generic_scan", "generic_output", "generic_chunk_dstate",
        "generic_reverse_scan", "generic_grad", "head_reduce", "mfma_state_scan_fwd", "mfma_output",
        "mfma_state_and_dstate_scans_bwd", "mfma_dstate_scan", "mfma_grad", "mfma_decay_prep", "mfma_vector_decay_prep", "mfma_vector_decay_dv", "recurrent_step",
        "walk_segment_summary", "walk_segment_scan", "walk_fwd", "walk_grad", "delta_prep", "delta_walk", "delta_reverse_walk", "delta_grad", "delta_segment_summary", "delta_segment_combine"};
    return kernel_id >= 0 && kernel_id < lsm::KID_COUNT ? names[kernel_id] : "unknown";
}

int lsm_kernel_path(const lsm_params* p) {
    lsm::Dims d{};
    const int rc = check_params(p, &d);
    if (rc != LSM_OK) return rc;
    return lsm::mfma_supported(d) ? 1 : 0;
}

namespace {
size_t fwd_bytes(const lsm::Dims& d) {
    return table_bytes(d) + (lsm::mfma_supported(d) ? lsm::mfma_fwd_workspace(d) : lsm::generic_fwd_workspace(d));
}
size_t bwd_bytes(const lsm::Dims& d) {
    return table_bytes(d) + (lsm::mfma_bwd_supported(d) ? lsm::mfma_bwd_workspace(d) : lsm::generic_bwd_workspace(d));
}
}  // namespace

// With LSM_FLAG_SAVE_STATES one buffer serves both calls, so both queries return the same figure.
int lsm_keeps_states(const lsm_params* p) {
    lsm::Dims d{};
    const int rc = check_params(p, &d);
    if (rc != LSM_OK) return rc;
    return d.save ? 1 : 0;
}

size_t lsm_chunk_fwd_workspace_bytes(const lsm_params* p) {
    lsm::Dims d{};
    if (check_params(p, &d) != LSM_OK) return 0;
    if (p->flags & LSM_FLAG_SAVE_STATES) return fwd_bytes(d) > bwd_bytes(d) ? fwd_bytes(d) : bwd_bytes(d);
    return fwd_bytes(d);
}

size_t lsm_chunk_bwd_workspace_bytes(const lsm_params* p) {
    lsm::Dims d{};
    if (check_params(p, &d) != LSM_OK) return 0;
    if (p->flags & LSM_FLAG_SAVE_STATES) return fwd_bytes(d) > bwd_bytes(d) ? fwd_bytes(d) : bwd_bytes(d);
    return bwd_bytes(d);
}

int lsm_chunk_fwd(const lsm_params* p, const void* q, const void* k, const void* v, const float* log_decay,
                  const float* init_state, void* o, float* final_state, void* workspace, size_t workspace_bytes,
                  void* stream) {
    lsm::Dims d{};
    const int rc = check_params(p, &d);
    if (rc != LSM_OK) return rc;
    if (!q || !k || !v || !o) return LSM_ERR_NULL;
    if ((d.kind == LSM_DECAY_NONE) != (log_decay == nullptr)) return LSM_ERR_NULL;
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(o) || misaligned(log_decay) ||
        misaligned(init_state) || misaligned(final_state) || misaligned(workspace))
        return LSM_ERR_ALIGN;
    const size_t need = lsm_chunk_fwd_workspace_bytes(p);
    if (!workspace || workspace_bytes < need) return LSM_ERR_WORKSPACE;
    if (prepare_tables(d, workspace, static_cast<hipStream_t>(stream)) != hipSuccess) return LSM_ERR_LAUNCH;
    lsm::FwdArgs a{q, k, v, log_decay, init_state, o, final_state, workspace, static_cast<hipStream_t>(stream)};
    const hipError_t e = lsm::mfma_supported(d) ? lsm::mfma_fwd(d, a) : lsm::generic_fwd(d, a);
    return e == hipSuccess ? LSM_OK : LSM_ERR_LAUNCH;
}

int lsm_chunk_fwd_noalloc(const lsm_params* p, const void* q, const void* k, const void* v, const float* log_decay,
                          const float* init_state, void* o, float* final_state, void* stream) {
    // every check of lsm_chunk_fwd, and the size limit, before the first HIP call
    lsm::Dims d{};
    const int rc = check_params(p, &d);
    if (rc != LSM_OK) return rc;
    if (!q || !k || !v || !o) return LSM_ERR_NULL;
    if ((d.kind == LSM_DECAY_NONE) != (log_decay == nullptr)) return LSM_ERR_NULL;
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(o) || misaligned(log_decay) ||
        misaligned(init_state) || misaligned(final_state))
        return LSM_ERR_ALIGN;
    if (lsm_chunk_fwd_workspace_bytes(p) > kScratchBytes) return LSM_ERR_WORKSPACE;
    void* ws = nullptr;
    if (scratch_of_current_device(&ws) != hipSuccess) return LSM_ERR_LAUNCH;
    return lsm_chunk_fwd(p, q, k, v, log_decay, init_state, o, final_state, ws, kScratchBytes, stream);
}

size_t lsm_bench_intra_chunk_workspace_bytes(const lsm_params* p) {
    lsm::Dims d{};
    if (check_params(p, &d) != LSM_OK || !lsm::mfma_supported(d) || d.kind == LSM_DECAY_VECTOR || d.nseq) return 0;
    return lsm::mfma_intra_bench_workspace(d);
}

int lsm_bench_intra_chunk(const lsm_params* p, const void* q, const void* k, const void* v, const float* log_decay,
                          void* o, void* workspace, size_t workspace_bytes, int repeats, void* stream) {
    lsm::Dims d{};
    const int rc = check_params(p, &d);
    if (rc != LSM_OK) return rc;
    if (!q || !k || !v || !o) return LSM_ERR_NULL;
    if ((d.kind == LSM_DECAY_NONE) != (log_decay == nullptr)) return LSM_ERR_NULL;
    if (!lsm::mfma_supported(d) || d.kind == LSM_DECAY_VECTOR || repeats < 1 || d.nseq) return LSM_ERR_UNSUPPORTED;
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(o) || misaligned(log_decay) || misaligned(workspace))
        return LSM_ERR_ALIGN;
    if (!workspace || workspace_bytes < lsm_bench_intra_chunk_workspace_bytes(p)) return LSM_ERR_WORKSPACE;
    lsm::FwdArgs a{q, k, v, log_decay, nullptr, o, nullptr, workspace, static_cast<hipStream_t>(stream)};
    return lsm::mfma_intra_bench(d, a, repeats) == hipSuccess ? LSM_OK : LSM_ERR_LAUNCH;
}

int lsm_step(const lsm_params* p, const void* q, const void* k, const void* v, const float* log_decay, float* state,
             void* o, void* stream) {
    lsm::Dims d{};
    const int rc = check_params(p, &d);
    if (rc != LSM_OK) return rc;
    if (!q || !k || !v || !o || !state) return LSM_ERR_NULL;
    if ((d.kind == LSM_DECAY_NONE) != (log_decay == nullptr)) return LSM_ERR_NULL;
    if (d.nseq) return LSM_ERR_UNSUPPORTED;  // one token per sequence: nothing to pack (the layout is immaterial for T = 1)
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(o) || misaligned(log_decay) || misaligned(state))
        return LSM_ERR_ALIGN;
    return lsm::step(d, q, k, v, log_decay, state, o, static_cast<hipStream_t>(stream)) == hipSuccess ? LSM_OK
                                                                                                    : LSM_ERR_LAUNCH;
}

int lsm_delta_step(const lsm_params* p, const void* q, const void* k, const void* v, const float* log_alpha, const float* beta,
                   const float* b, float* state, void* o, void* stream) {
    lsm::Dims d{};
    const int rc = check_params(p, &d);
    if (rc != LSM_OK) return rc;
    if (!q || !k || !v || !o || !state) return LSM_ERR_NULL;
    if (d.kind != LSM_DECAY_NONE && d.kind != LSM_DECAY_SCALAR) return LSM_ERR_UNSUPPORTED;
    if ((d.kind == LSM_DECAY_NONE) != (log_alpha == nullptr)) return LSM_ERR_NULL;
    if (d.nseq) return LSM_ERR_UNSUPPORTED;
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(o) || misaligned(log_alpha) || misaligned(beta) ||
        misaligned(b) || misaligned(state))
        return LSM_ERR_ALIGN;
    return lsm::delta_step(d, q, k, v, log_alpha, beta, b, state, o, static_cast<hipStream_t>(stream)) == hipSuccess
               ? LSM_OK : LSM_ERR_LAUNCH;
}

size_t lsm_delta_fwd_workspace_bytes(const lsm_params* p) {
    lsm::Dims d{};
    if (check_params(p, &d) != LSM_OK || !lsm::delta_supported(d)) return 0;
    d.save = (p->flags & LSM_FLAG_SAVE_STATES) != 0;
    return table_bytes(d) + lsm::delta_fwd_workspace(d);
}

int lsm_delta_fwd(const lsm_params* p, const void* q, const void* k, const void* v, const float* log_alpha,
                  const float* beta, const float* b, const float* init_state, void* o, float* final_state,
                  void* workspace, size_t workspace_bytes, void* stream) {
    lsm::Dims d{};
    const int rc = check_params(p, &d);
    if (rc != LSM_OK) return rc;
    if (!q || !k || !v || !o) return LSM_ERR_NULL;
    if (d.kind != LSM_DECAY_NONE && d.kind != LSM_DECAY_SCALAR) return LSM_ERR_UNSUPPORTED;
    if ((d.kind == LSM_DECAY_NONE) != (log_alpha == nullptr)) return LSM_ERR_NULL;
    if (!lsm::delta_supported(d)) return LSM_ERR_UNSUPPORTED;
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(o) || misaligned(log_alpha) || misaligned(beta) ||
        misaligned(b) || misaligned(init_state) || misaligned(final_state) || misaligned(workspace))
        return LSM_ERR_ALIGN;
    d.save = (p->flags & LSM_FLAG_SAVE_STATES) != 0;
    if (!workspace || workspace_bytes < table_bytes(d) + lsm::delta_fwd_workspace(d)) return LSM_ERR_WORKSPACE;
    if (prepare_tables(d, workspace, static_cast<hipStream_t>(stream)) != hipSuccess) return LSM_ERR_LAUNCH;
    const lsm::DeltaArgs a{q, k, v, log_alpha, beta, b, init_state, o, final_state, workspace, static_cast<hipStream_t>(stream)};
    return lsm::delta_fwd(d, a) == hipSuccess ? LSM_OK : LSM_ERR_LAUNCH;
}

size_t lsm_delta_bwd_workspace_bytes(const lsm_params* p) {
    lsm::Dims d{};
    if (check_params(p, &d) != LSM_OK || !lsm::delta_supported(d)) return 0;
    return table_bytes(d) + lsm::delta_bwd_workspace(d);
}

int lsm_delta_bwd(const lsm_params* p, const void* q, const void* k, const void* v, const float* log_alpha,
                  const float* beta, const float* b, const float* init_state, const void* d_o,
                  const float* d_final_state, void* dq, void* dk, void* dv, float* d_log_alpha, float* d_beta, float* d_b,
                  float* d_init_state, void* workspace, size_t workspace_bytes, void* stream) {
    lsm::Dims d{};
    const int rc = check_params(p, &d);
    if (rc != LSM_OK) return rc;
    if (!q || !k || !v || !d_o || !dq || !dk || !dv) return LSM_ERR_NULL;
    if (d.kind != LSM_DECAY_NONE && d.kind != LSM_DECAY_SCALAR) return LSM_ERR_UNSUPPORTED;
    if ((d.kind == LSM_DECAY_NONE) != (log_alpha == nullptr)) return LSM_ERR_NULL;
    // a gradient is wanted exactly for the parameters that were given
    if ((log_alpha == nullptr) != (d_log_alpha == nullptr) || (beta == nullptr) != (d_beta == nullptr) ||
        (b == nullptr) != (d_b == nullptr))
        return LSM_ERR_NULL;
    if (!lsm::delta_supported(d)) return LSM_ERR_UNSUPPORTED;
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(d_o) || misaligned(dq) || misaligned(dk) ||
        misaligned(dv) || misaligned(log_alpha) || misaligned(beta) || misaligned(b) || misaligned(init_state) ||
        misaligned(d_final_state) || misaligned(d_log_alpha) || misaligned(d_beta) || misaligned(d_b) ||
        misaligned(d_init_state) || misaligned(workspace))
        return LSM_ERR_ALIGN;
    d.save = (p->flags & LSM_FLAG_SAVE_STATES) != 0;
    if (!workspace || workspace_bytes < table_bytes(d) + lsm::delta_bwd_workspace(d)) return LSM_ERR_WORKSPACE;
    if (prepare_tables(d, workspace, static_cast<hipStream_t>(stream)) != hipSuccess) return LSM_ERR_LAUNCH;
    const lsm::DeltaBwdArgs a{q, k, v, log_alpha, beta, b, init_state, d_o, d_final_state, dq, dk, dv, d_log_alpha, d_beta, d_b,
                              d_init_state, workspace, static_cast<hipStream_t>(stream)};
    return lsm::delta_bwd(d, a) == hipSuccess ? LSM_OK : LSM_ERR_LAUNCH;
}

int lsm_chunk_bwd(const lsm_params* p, const void* q, const void* k, const void* v, const float* log_decay,
                  const float* init_state, const void* d_o, const float* d_final_state, void* dq, void* dk,
                  void* dv, float* d_log_decay, float* d_init_state, void* workspace, size_t workspace_bytes,
                  void* stream) {
    lsm::Dims d{};
    const int rc = check_params(p, &d);
    if (rc != LSM_OK) return rc;
    if (!q || !k || !v || !d_o || !dq || !dk || !dv) return LSM_ERR_NULL;
    if ((d.kind == LSM_DECAY_NONE) != (log_decay == nullptr)) return LSM_ERR_NULL;
    if (d.kind == LSM_DECAY_NONE && d_log_decay) return LSM_ERR_NULL;
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(d_o) || misaligned(dq) || misaligned(dk) ||
        misaligned(dv) || misaligned(log_decay) || misaligned(init_state) || misaligned(d_final_state) ||
        misaligned(d_log_decay) || misaligned(d_init_state) || misaligned(workspace))
        return LSM_ERR_ALIGN;
    const size_t need = lsm_chunk_bwd_workspace_bytes(p);
    if (!workspace || workspace_bytes < need) return LSM_ERR_WORKSPACE;
    if (prepare_tables(d, workspace, static_cast<hipStream_t>(stream)) != hipSuccess) return LSM_ERR_LAUNCH;
    lsm::BwdArgs a{q, k, v, log_decay, init_state, d_o, d_final_state, dq, dk, dv, d_log_decay, d_init_state,
                   workspace, static_cast<hipStream_t>(stream)};
    const hipError_t e = lsm::mfma_bwd_supported(d) ? lsm::mfma_bwd(d, a) : lsm::generic_bwd(d, a);
    return e == hipSuccess ? LSM_OK : LSM_ERR_LAUNCH;
}

}  // extern "C"
