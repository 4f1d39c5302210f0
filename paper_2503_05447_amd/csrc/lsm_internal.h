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

// Generic family: fp32 arithmetic on plain ALU, every supported shape, both element types.
size_t generic_fwd_workspace(const Dims& d);
size_t generic_bwd_workspace(const Dims& d);
hipError_t generic_fwd(const Dims& d, const FwdArgs& a);
hipError_t generic_bwd(const Dims& d, const BwdArgs& a);

// MFMA family: bf16 operands, fp32 accumulation, for the shapes mfma_supported() accepts.
bool mfma_supported(const Dims& d);
size_t mfma_fwd_workspace(const Dims& d);
size_t mfma_bwd_workspace(const Dims& d);
hipError_t mfma_fwd(const Dims& d, const FwdArgs& a);
hipError_t mfma_bwd(const Dims& d, const BwdArgs& a);

}  // namespace lsm
