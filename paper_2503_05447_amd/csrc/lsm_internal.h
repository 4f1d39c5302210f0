// Internal declarations shared by the kernels and the C-ABI front end of the
// gfx950 LSM library.  Nothing here is visible to callers.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace lsm {

// Problem geometry handed to every launcher.  N = ceil(T / C) chunks per sequence.
struct Dims {
    int B, H, T, dk, dv, C, N, kind;
    bool bf16;  // element type of q,k,v,o and their gradients
    __host__ __device__ int BH() const { return B * H; }
    __host__ __device__ int dkd() const { return kind == 3 ? dk : 1; }  // decay values per token
};

// Pointers of one forward call (device memory).
struct FwdArgs {
    const void *q, *k, *v;
    const float *g, *m0;
    void* o;
    float* mT;
    void* ws;
    hipStream_t stream;
};

// Pointers of one backward call (device memory).
struct BwdArgs {
    const void *q, *k, *v;
    const float *g, *m0;
    const void* d_o;
    const float* d_mT;
    void *dq, *dk, *dv;
    float *dg, *d_m0;
    void* ws;
    hipStream_t stream;
};

inline size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

// Kernel identifiers reported by the optional per-kernel timing (lsm_profile_start / _stop).
enum KernelId {
    KID_GEN_CUMSUM = 0, KID_GEN_STATE, KID_GEN_SCAN, KID_GEN_OUTPUT, KID_GEN_DSTATE, KID_GEN_RSCAN, KID_GEN_GRAD,
    KID_HEAD_REDUCE, KID_MFMA_STATE, KID_MFMA_OUTPUT, KID_MFMA_STATE_BWD, KID_MFMA_DSTATE, KID_MFMA_GRAD, KID_MFMA_PREP, KID_MFMA_VEC_PREP, KID_MFMA_VEC_DV, KID_STEP, KID_COUNT
};
// Bracket a kernel launch with events when timing is switched on (no-ops otherwise).
void prof_begin(int kernel_id, hipStream_t stream);
void prof_end(hipStream_t stream);
struct ProfScope {
    hipStream_t s;
    ProfScope(int id, hipStream_t stream) : s(stream) { prof_begin(id, stream); }
    ~ProfScope() { prof_end(s); }
};

// Generic family: fp32 arithmetic on plain ALU, every supported shape, both element types.
size_t generic_fwd_workspace(const Dims& d);
size_t generic_bwd_workspace(const Dims& d);
hipError_t generic_fwd(const Dims& d, const FwdArgs& a);
hipError_t generic_bwd(const Dims& d, const BwdArgs& a);

// MFMA family: bf16 operands, fp32 accumulation, for the shapes mfma_supported() accepts.
bool mfma_supported(const Dims& d);      // forward
bool mfma_bwd_supported(const Dims& d);  // backward
size_t mfma_fwd_workspace(const Dims& d);
size_t mfma_bwd_workspace(const Dims& d);
hipError_t mfma_fwd(const Dims& d, const FwdArgs& a);
hipError_t mfma_bwd(const Dims& d, const BwdArgs& a);
// benchmark aid: the output kernel alone with its compute phase repeated `reps` times (scalar decay kinds);
// the workspace must hold the chunk states of a preceding mfma_fwd call on the same inputs
hipError_t mfma_intra_bench(const Dims& d, const FwdArgs& a, int reps);

// Recurrent single-token step (decoding): state updated in place, T of the Dims ignored.
hipError_t step(const Dims& d, const void* q, const void* k, const void* v, const float* g, float* state, void* o,
                hipStream_t stream);

}  // namespace lsm
