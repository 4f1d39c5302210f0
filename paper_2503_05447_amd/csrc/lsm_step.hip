// Recurrent single-token step of the LSM recurrence (Eq. 5 with the rank-1 update of Table 1), the
// constant-memory form used for decoding:
//     M <- diag(a) M + k^T v ,   o = q M          per (b,h), M in fp32 [d_k][d_v], updated in place.
// The step moves 8 d_k d_v bytes of state per head and does 4 d_k d_v flops on them: it is bound by
// HBM.  A workgroup owns a strip of 64 state columns of one (b,h): 16 row groups x 16 column groups
// of threads, each thread d_k/16 rows x 4 columns (16-byte accesses, whole 256-byte row pieces per 16
// lanes), all loads of a thread issued before the first use; the partial outputs of the 16 row groups
// are summed in a fixed order through LDS.  Ordinary (cacheable) accesses: the state is read again by
// the next step, and for serving batches it fits the memory-side cache.
#include "lsm_internal.h"

namespace lsm {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float elem(const float* p, size_t i) { return p[i]; }
__device__ __forceinline__ float elem(const uint16_t* p, size_t i) { return __uint_as_float(uint32_t(p[i]) << 16); }
__device__ __forceinline__ void put(float* p, size_t i, float x) { p[i] = x; }
__device__ __forceinline__ void put(uint16_t* p, size_t i, float x) {
    uint32_t u = __float_as_uint(x);
    if ((u & 0x7fffffffu) > 0x7f800000u) { p[i] = uint16_t((u >> 16) | 0x40); return; }
    u += 0x7fffu + ((u >> 16) & 1u);  // round to nearest even
    p[i] = uint16_t(u >> 16);
}

template <typename TIO, int DK>
__global__ __launch_bounds__(256) void k_step(Dims d, const TIO* __restrict__ q, const TIO* __restrict__ k,
                                              const TIO* __restrict__ v, const float* __restrict__ g,
                                              float* __restrict__ state, TIO* __restrict__ o) {
    constexpr int R = DK / 16;  // rows per thread
    __shared__ float part[16][64];
    const int bh = blockIdx.y, col0 = 64 * blockIdx.x, tid = threadIdx.x;
    const int cg = tid & 15, rg = tid >> 4, h = bh % d.H;
    float* M = state + size_t(bh) * DK * d.dv + col0 + 4 * cg;
    f32x4 m[R];
    _Pragma("unroll") for (int r = 0; r < R; ++r)
        m[r] = *reinterpret_cast<const f32x4*>(M + size_t(rg + 16 * r) * d.dv);
    float vv[4];
    _Pragma("unroll") for (int c = 0; c < 4; ++c) vv[c] = elem(v, size_t(bh) * d.dv + col0 + 4 * cg + c);
    const float gs = d.kind == 1 ? g[h] : (d.kind == 2 ? g[bh] : 0.f);
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    _Pragma("unroll") for (int r = 0; r < R; ++r) {
        const int i = rg + 16 * r;
        const float a = d.kind == 0 ? 1.f : expf(d.kind == 3 ? g[size_t(bh) * DK + i] : gs);
        const float ki = elem(k, size_t(bh) * DK + i), qi = elem(q, size_t(bh) * DK + i);
        _Pragma("unroll") for (int c = 0; c < 4; ++c) {
            m[r][c] = a * m[r][c] + ki * vv[c];
            acc[c] += qi * m[r][c];
        }
        *reinterpret_cast<f32x4*>(M + size_t(i) * d.dv) = m[r];
    }
    _Pragma("unroll") for (int c = 0; c < 4; ++c) part[rg][4 * cg + c] = acc[c];
    __syncthreads();
    if (tid < 64) {
        float s = 0.f;
        _Pragma("unroll") for (int r = 0; r < 16; ++r) s += part[r][tid];
        put(o, size_t(bh) * d.dv + col0 + tid, s);
    }
}

// The same step for the delta-rule rows of Table 1 (DeltaNet, Gated DeltaNet):
//     M <- alpha (M - beta k^T (k M)) + b k^T v ,   o = q M .
// The erase term needs w = k M over all rows before any row changes: the strip's partial sums of w go through LDS
// first (the state stays in registers meanwhile), then the update and the read-out as above.
template <typename TIO, int DK>
__global__ __launch_bounds__(256) void k_delta_step(Dims d, const TIO* __restrict__ q, const TIO* __restrict__ k,
                                                    const TIO* __restrict__ v, const float* __restrict__ log_alpha,
                                                    const float* __restrict__ beta, const float* __restrict__ bw,
                                                    float* __restrict__ state, TIO* __restrict__ o) {
    constexpr int R = DK / 16;
    __shared__ float part[16][64];
    __shared__ float wsum[64];
    const int bh = blockIdx.y, col0 = 64 * blockIdx.x, tid = threadIdx.x;
    const int cg = tid & 15, rg = tid >> 4;
    float* M = state + size_t(bh) * DK * d.dv + col0 + 4 * cg;
    f32x4 m[R];
    _Pragma("unroll") for (int r = 0; r < R; ++r)
        m[r] = *reinterpret_cast<const f32x4*>(M + size_t(rg + 16 * r) * d.dv);
    float vv[4], ki[R], qi[R];
    _Pragma("unroll") for (int c = 0; c < 4; ++c) vv[c] = elem(v, size_t(bh) * d.dv + col0 + 4 * cg + c);
    const float al = log_alpha ? expf(log_alpha[bh]) : 1.f, be = beta ? beta[bh] : 1.f, b_ = bw ? bw[bh] : 1.f;
    f32x4 w = {0.f, 0.f, 0.f, 0.f};
    _Pragma("unroll") for (int r = 0; r < R; ++r) {
        const int i = rg + 16 * r;
        ki[r] = elem(k, size_t(bh) * DK + i);
        qi[r] = elem(q, size_t(bh) * DK + i);
        _Pragma("unroll") for (int c = 0; c < 4; ++c) w[c] += ki[r] * m[r][c];
    }
    _Pragma("unroll") for (int c = 0; c < 4; ++c) part[rg][4 * cg + c] = w[c];
    __syncthreads();
    if (tid < 64) {
        float s = 0.f;
        _Pragma("unroll") for (int r = 0; r < 16; ++r) s += part[r][tid];
        wsum[tid] = s;
    }
    __syncthreads();
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    _Pragma("unroll") for (int r = 0; r < R; ++r) {
        const int i = rg + 16 * r;
        _Pragma("unroll") for (int c = 0; c < 4; ++c) {
            m[r][c] = al * (m[r][c] - be * ki[r] * wsum[4 * cg + c]) + b_ * ki[r] * vv[c];
            acc[c] += qi[r] * m[r][c];
        }
        *reinterpret_cast<f32x4*>(M + size_t(i) * d.dv) = m[r];
    }
    _Pragma("unroll") for (int c = 0; c < 4; ++c) part[rg][4 * cg + c] = acc[c];
    __syncthreads();
    if (tid < 64) {
        float s = 0.f;
        _Pragma("unroll") for (int r = 0; r < 16; ++r) s += part[r][tid];
        put(o, size_t(bh) * d.dv + col0 + tid, s);
    }
}

template <typename TIO>
hipError_t launch_delta(const Dims& d, const void* q, const void* k, const void* v, const float* la, const float* be,
                        const float* bw, float* state, void* o, hipStream_t st) {
    const dim3 grid(d.dv / 64, d.BH()), block(256);
    auto Q = static_cast<const TIO*>(q), K = static_cast<const TIO*>(k), V = static_cast<const TIO*>(v);
    auto O = static_cast<TIO*>(o);
    ProfScope ps(KID_STEP, st);
    if (d.dk == 64) hipLaunchKernelGGL((k_delta_step<TIO, 64>), grid, block, 0, st, d, Q, K, V, la, be, bw, state, O);
    else if (d.dk == 128) hipLaunchKernelGGL((k_delta_step<TIO, 128>), grid, block, 0, st, d, Q, K, V, la, be, bw, state, O);
    else hipLaunchKernelGGL((k_delta_step<TIO, 256>), grid, block, 0, st, d, Q, K, V, la, be, bw, state, O);
    return hipGetLastError();
}

template <typename TIO>
hipError_t launch(const Dims& d, const void* q, const void* k, const void* v, const float* g, float* state, void* o,
                  hipStream_t st) {
    const dim3 grid(d.dv / 64, d.BH()), block(256);
    auto Q = static_cast<const TIO*>(q), K = static_cast<const TIO*>(k), V = static_cast<const TIO*>(v);
    auto O = static_cast<TIO*>(o);
    ProfScope ps(KID_STEP, st);
    if (d.dk == 64) hipLaunchKernelGGL((k_step<TIO, 64>), grid, block, 0, st, d, Q, K, V, g, state, O);
    else if (d.dk == 128) hipLaunchKernelGGL((k_step<TIO, 128>), grid, block, 0, st, d, Q, K, V, g, state, O);
    else hipLaunchKernelGGL((k_step<TIO, 256>), grid, block, 0, st, d, Q, K, V, g, state, O);
    return hipGetLastError();
}

}  // namespace

hipError_t step(const Dims& d, const void* q, const void* k, const void* v, const float* g, float* state, void* o,
                hipStream_t st) {
    return d.bf16 ? launch<uint16_t>(d, q, k, v, g, state, o, st) : launch<float>(d, q, k, v, g, state, o, st);
}

hipError_t delta_step(const Dims& d, const void* q, const void* k, const void* v, const float* log_alpha, const float* beta,
                      const float* bw, float* state, void* o, hipStream_t st) {
    return d.bf16 ? launch_delta<uint16_t>(d, q, k, v, log_alpha, beta, bw, state, o, st)
                  : launch_delta<float>(d, q, k, v, log_alpha, beta, bw, state, o, st);
}

}  // namespace lsm
