// Generic kernel family of the chunkwise LSM path: fp32 arithmetic on the plain
// vector ALU, any supported (d_k, d_v, chunk) and both element types.  It is
// the product path for fp32 inputs (whose 1e-4 tolerance rules out bf16 MFMA
// operands) and for shapes the MFMA family does not cover.
//
// Structure (Algorithm 2 of the paper, generalised to a decay):
//   cumsum      b_j  = chunk-local inclusive sum of the log-decay
//   local_state U_c  = sum_r (k_r * e^{b_C - b_r})^T v_r             (Alg. 2: M_t = K_t^T V_t)
//   scan        S_{c+1} = diag(e^{b_C}) S_c + U_c                     (Alg. 2: PrefixSum)
//   output      O = [(Q K^T) * D * Psi] V + (Q * e^{b}) S_c            (Alg. 2: O_intra + O_inter)
// and for the backward the mirrored dU / reverse scan / per-chunk gradients.
#include "lsm_internal.h"

namespace lsm {
namespace {

constexpr int kThreads = 256;

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(uint16_t x) { return __uint_as_float(uint32_t(x) << 16); }

__device__ __forceinline__ void from_f32(float* p, float x) { *p = x; }
__device__ __forceinline__ void from_f32(uint16_t* p, float x) {
    // round to nearest even; inputs are finite by contract, NaN is kept quiet
    uint32_t u = __float_as_uint(x);
    if ((u & 0x7fffffffu) > 0x7f800000u) { *p = uint16_t((u >> 16) | 0x40); return; }
    u += 0x7fffu + ((u >> 16) & 1u);
    *p = uint16_t(u >> 16);
}

// Chunk-local cumulative log-decay of token `tok` (= bh*T + t), feature i.  Kept in fp64: the sums
// reach hundreds for strong decays while only their O(1) differences enter exp(), and an fp32 sum
// would leave ~1e-4 relative error in those, which is the whole budget of the fp32 path.
using bsum_t = double;
__device__ __forceinline__ bsum_t bval(const bsum_t* bcum, size_t tok, int dkd, int i) {
    return bcum ? bcum[tok * dkd + (dkd > 1 ? i : 0)] : 0.0;
}
__device__ __forceinline__ float expd(bsum_t x) { return expf(float(x)); }

// ---------------------------------------------------------------------------------------------
// b_j = sum_{r<=j, r in chunk} g_r   (grid: N x BH)
__global__ void k_cumsum(Dims d, const float* __restrict__ g, bsum_t* __restrict__ bcum) {
    const int c = blockIdx.x, bh = blockIdx.y, h = bh % d.H;
    const ChunkPos cp = chunk_pos(d, c, bh);
    const int L = cp.L, dkd = d.dkd();
    for (int i = threadIdx.x; i < dkd; i += blockDim.x) {
        bsum_t b = 0.0;
        for (int j = 0; j < L; ++j) {
            const size_t tok = cp.tok0 + size_t(j) * cp.ts;  // in the caller's arrays
            float gv = d.kind == 1 ? g[h] : (d.kind == 2 ? g[tok] : g[tok * d.dk + i]);
            b += gv;
            bcum[(cp.wtok0 + j) * dkd + i] = b;
        }
    }
}

// MODE 0:  out_c = sum_r (x_r * e^{b_C - b_r})^T y_r      (x = k, y = v : chunk state U_c)
// MODE 1:  out_c = sum_j (x_j * e^{b_j})^T y_j            (x = q, y = d_o : chunk state gradient dU_c)
template <typename TIO, int MODE>
__global__ void k_local_state(Dims d, const TIO* __restrict__ x, const TIO* __restrict__ y,
                              const bsum_t* __restrict__ bcum, float* __restrict__ out) {
    const int c = blockIdx.x, bh = blockIdx.y;
    const ChunkPos cp = chunk_pos(d, c, bh);
    const int L = cp.L, dkd = d.dkd();
    if (L <= 0) return;  // packed input: the grid is sized for an upper bound of the chunk count
    const size_t tok0 = cp.wtok0;                              // token index in the library's own arrays
    auto U = [&](int r) { return cp.tok0 + size_t(r) * cp.ts; };  // row of token r in the caller's arrays
    float* dst = out + cp.slot * d.dk * d.dv;
    // scalar kinds: the weight depends on the token only, one table per chunk instead of an exp per product
    __shared__ float wtok[128];
    if (dkd == 1) {
        const bsum_t bC = bval(bcum, tok0 + L - 1, 1, 0);
        for (int r = threadIdx.x; r < L; r += blockDim.x) {
            const bsum_t br = bval(bcum, tok0 + r, 1, 0);
            wtok[r] = MODE == 0 ? expd(bC - br) : expd(br);
        }
        __syncthreads();
    }
    for (int e = threadIdx.x; e < d.dk * d.dv; e += blockDim.x) {
        const int i = e / d.dv, j = e % d.dv;
        float acc = 0.f;
        if (dkd == 1) {
            _Pragma("unroll 8")
            for (int r = 0; r < L; ++r) acc += to_f32(x[U(r) * d.dk + i]) * wtok[r] * to_f32(y[U(r) * d.dv + j]);
        } else {
            const bsum_t bC = bval(bcum, tok0 + L - 1, dkd, i);
            for (int r = 0; r < L; ++r) {
                const bsum_t br = bval(bcum, tok0 + r, dkd, i);
                const float w = MODE == 0 ? expd(bC - br) : expd(br);
                acc += to_f32(x[U(r) * d.dk + i]) * w * to_f32(y[U(r) * d.dv + j]);
            }
        }
        dst[e] = acc;
    }
}

// Forward scan over chunks, in place: slot c holds U_c on entry and S_c (state at the START of
// chunk c) on exit; S_{c+1} = e^{b_C} * S_c + U_c.   REVERSE: slot c holds dU_c on entry and
// dS_{c+1} (gradient w.r.t. the state at the END of chunk c) on exit; dS_c = e^{b_C} * dS_{c+1} + dU_c.
// `edge_in` is M_0 (or d M_T), `edge_out` receives M_T (or d M_0); either may be NULL.
template <bool REVERSE>
__global__ void k_scan(Dims d, const bsum_t* __restrict__ bcum, float* __restrict__ states,
                       const float* __restrict__ edge_in, float* __restrict__ edge_out) {
    const SeqWalk w = seq_walk(d, blockIdx.y);  // grid.y = Dims::seqs()
    const int dkd = d.dkd();
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    const int sz = d.dk * d.dv;
    if (e >= sz) return;
    const int i = e / d.dv;
    float s = edge_in ? edge_in[size_t(w.edge) * sz + e] : 0.f;
    for (int n = 0; n < w.n; ++n) {
        const ChunkPos cp = walk_pos(d, w, REVERSE ? w.n - 1 - n : n);
        const float lam = expd(bval(bcum, cp.wtok0 + cp.L - 1, dkd, i));
        float* slot = states + cp.slot * sz + e;
        const float u = *slot;
        *slot = s;
        s = lam * s + u;
    }
    if (edge_out) edge_out[size_t(w.edge) * sz + e] = s;
}

// A_jr = sum_i q_ji k_ri e^{b_ji - b_ri}  for r <= j  (0 otherwise), into LDS [C*C]
template <typename TIO>
__device__ void scores_to_lds(const Dims& d, const TIO* q, const TIO* k, const bsum_t* bcum, const ChunkPos& cp,
                              int L, float* A) {
    const int dkd = d.dkd();
    const size_t tok0 = cp.wtok0;
    auto U = [&](int r) { return cp.tok0 + size_t(r) * cp.ts; };
    for (int e = threadIdx.x; e < L * L; e += blockDim.x) {
        const int j = e / L, r = e % L;
        float acc = 0.f;
        if (r <= j) {
            if (dkd == 1) {
                _Pragma("unroll 8")
                for (int i = 0; i < d.dk; ++i)
                    acc += to_f32(q[U(j) * d.dk + i]) * to_f32(k[U(r) * d.dk + i]);
                acc *= expd(bval(bcum, tok0 + j, 1, 0) - bval(bcum, tok0 + r, 1, 0));
            } else {
                for (int i = 0; i < d.dk; ++i)
                    acc += to_f32(q[U(j) * d.dk + i]) * to_f32(k[U(r) * d.dk + i]) *
                           expd(bcum[(tok0 + j) * dkd + i] - bcum[(tok0 + r) * dkd + i]);
            }
        }
        A[j * d.C + r] = acc;
    }
}

// o_j = sum_{r<=j} A_jr v_r + (q_j * e^{b_j}) S_c      (grid: N x BH, dynamic LDS C*C floats)
template <typename TIO>
__global__ void k_output(Dims d, const TIO* __restrict__ q, const TIO* __restrict__ k, const TIO* __restrict__ v,
                         const bsum_t* __restrict__ bcum, const float* __restrict__ states, TIO* __restrict__ o) {
    extern __shared__ float lds[];
    float* A = lds;
    const int c = blockIdx.x, bh = blockIdx.y;
    const ChunkPos cp = chunk_pos(d, c, bh);
    const int L = cp.L, dkd = d.dkd();
    if (L <= 0) return;  // packed input: the grid is sized for an upper bound of the chunk count
    const size_t tok0 = cp.wtok0;                              // token index in the library's own arrays
    auto U = [&](int r) { return cp.tok0 + size_t(r) * cp.ts; };  // row of token r in the caller's arrays
    const float* S = states + cp.slot * d.dk * d.dv;
    scores_to_lds(d, q, k, bcum, cp, L, A);
    __syncthreads();
    for (int e = threadIdx.x; e < L * d.dv; e += blockDim.x) {
        const int j = e / d.dv, col = e % d.dv;
        float acc = 0.f;
        _Pragma("unroll 8")
        for (int r = 0; r <= j; ++r) acc += A[j * d.C + r] * to_f32(v[U(r) * d.dv + col]);
        if (dkd == 1) {  // one decay factor per token
            float inter = 0.f;
            _Pragma("unroll 8")
            for (int i = 0; i < d.dk; ++i) inter += to_f32(q[U(j) * d.dk + i]) * S[i * d.dv + col];
            acc += expd(bval(bcum, tok0 + j, 1, 0)) * inter;
        } else {
            for (int i = 0; i < d.dk; ++i)
                acc += to_f32(q[U(j) * d.dk + i]) * expd(bval(bcum, tok0 + j, dkd, i)) * S[i * d.dv + col];
        }
        from_f32(&o[U(j) * d.dv + col], acc);
    }
}

// Per-chunk gradients (grid: N x BH, dynamic LDS 2*C*C floats).
//   dA_jr = d_o_j . v_r                                    (r <= j)
//   dq_j  = e^{b_j} * (d_o_j S_c^T)            + sum_{r<=j} dA_jr e^{b_j-b_r} * k_r
//   dk_r  = e^{b_C-b_r} * (v_r dS_{c+1}^T)     + sum_{j>=r} dA_jr e^{b_j-b_r} * q_j
//   dv_r  = (k_r * e^{b_C-b_r}) dS_{c+1}       + sum_{j>=r} A_jr d_o_j
//   dg_t  = sum_{u>=t in chunk} (q_u*dq_u - k_u*dk_u) + sum_{r in chunk} k_r*dk_r^{inter}
//           + e^{b_C} * rowsum(S_c * dS_{c+1})
// wq / wk: fp32 scratch [BH,T,dk] each; dg_tok: [BH,T] scratch for the per-head kind.
template <typename TIO>
__global__ void k_grad(Dims d, const TIO* __restrict__ q, const TIO* __restrict__ k, const TIO* __restrict__ v,
                       const TIO* __restrict__ d_o, const bsum_t* __restrict__ bcum,
                       const float* __restrict__ states, const float* __restrict__ dstates,
                       TIO* __restrict__ dq, TIO* __restrict__ dk, TIO* __restrict__ dv,
                       float* __restrict__ dg, float* __restrict__ wq, float* __restrict__ wk,
                       float* __restrict__ dg_tok) {
    extern __shared__ float lds[];
    float* A = lds;
    float* dA = lds + d.C * d.C;
    const int c = blockIdx.x, bh = blockIdx.y;
    const ChunkPos cp = chunk_pos(d, c, bh);
    const int L = cp.L, dkd = d.dkd();
    if (L <= 0) return;  // packed input: the grid is sized for an upper bound of the chunk count
    const size_t tok0 = cp.wtok0;                              // token index in the library's own arrays
    auto U = [&](int r) { return cp.tok0 + size_t(r) * cp.ts; };  // row of token r in the caller's arrays
    const float* S = states + cp.slot * d.dk * d.dv;
    const float* dS = dstates + cp.slot * d.dk * d.dv;
    const bool want_dg = dg != nullptr || dg_tok != nullptr;

    scores_to_lds(d, q, k, bcum, cp, L, A);
    for (int e = threadIdx.x; e < L * L; e += blockDim.x) {
        const int j = e / L, r = e % L;
        float acc = 0.f;
        if (r <= j)
            _Pragma("unroll 8")
            for (int col = 0; col < d.dv; ++col)
                acc += to_f32(d_o[U(j) * d.dv + col]) * to_f32(v[U(r) * d.dv + col]);
        // scalar kinds: the decay of a score depends on the token pair only, so G = dA * D is formed here
        // once and the loops below contain no exponential
        if (dkd == 1 && r <= j) acc *= expd(bval(bcum, tok0 + j, 1, 0) - bval(bcum, tok0 + r, 1, 0));
        dA[j * d.C + r] = acc;
    }
    __syncthreads();

    // dv
    for (int e = threadIdx.x; e < L * d.dv; e += blockDim.x) {
        const int r = e / d.dv, col = e % d.dv;
        float acc = 0.f;
        _Pragma("unroll 8")
        for (int j = r; j < L; ++j) acc += A[j * d.C + r] * to_f32(d_o[U(j) * d.dv + col]);
        if (dkd == 1) {  // one decay factor per token
            float inter = 0.f;
            _Pragma("unroll 8")
            for (int i = 0; i < d.dk; ++i) inter += to_f32(k[U(r) * d.dk + i]) * dS[i * d.dv + col];
            acc += expd(bval(bcum, tok0 + L - 1, 1, 0) - bval(bcum, tok0 + r, 1, 0)) * inter;
        } else {
            for (int i = 0; i < d.dk; ++i) {
                const float w = expd(bval(bcum, tok0 + L - 1, dkd, i) - bval(bcum, tok0 + r, dkd, i));
                acc += to_f32(k[U(r) * d.dk + i]) * w * dS[i * d.dv + col];
            }
        }
        from_f32(&dv[U(r) * d.dv + col], acc);
    }
    // dq, dk and the per-token terms of the decay gradient
    for (int e = threadIdx.x; e < L * d.dk; e += blockDim.x) {
        const int t = e / d.dk, i = e % d.dk;
        const bsum_t bt = bval(bcum, tok0 + t, dkd, i);
        const bsum_t bC = bval(bcum, tok0 + L - 1, dkd, i);
        float q_inter = 0.f, k_inter = 0.f;
        _Pragma("unroll 8")
        for (int col = 0; col < d.dv; ++col) {
            q_inter += to_f32(d_o[U(t) * d.dv + col]) * S[i * d.dv + col];
            k_inter += to_f32(v[U(t) * d.dv + col]) * dS[i * d.dv + col];
        }
        q_inter *= expd(bt);
        k_inter *= expd(bC - bt);
        float q_intra = 0.f, k_intra = 0.f;
        if (dkd == 1) {  // dA already carries the decay
            _Pragma("unroll 8")
            for (int r = 0; r <= t; ++r) q_intra += dA[t * d.C + r] * to_f32(k[U(r) * d.dk + i]);
            _Pragma("unroll 8")
            for (int j = t; j < L; ++j) k_intra += dA[j * d.C + t] * to_f32(q[U(j) * d.dk + i]);
        } else {
            for (int r = 0; r <= t; ++r)
                q_intra += dA[t * d.C + r] * expd(bt - bval(bcum, tok0 + r, dkd, i)) * to_f32(k[U(r) * d.dk + i]);
            for (int j = t; j < L; ++j)
                k_intra += dA[j * d.C + t] * expd(bval(bcum, tok0 + j, dkd, i) - bt) * to_f32(q[U(j) * d.dk + i]);
        }
        const float dqv = q_inter + q_intra, dkv = k_inter + k_intra;
        from_f32(&dq[U(t) * d.dk + i], dqv);
        from_f32(&dk[U(t) * d.dk + i], dkv);
        if (want_dg) {
            const float qv = to_f32(q[U(t) * d.dk + i]), kv = to_f32(k[U(t) * d.dk + i]);
            wq[(tok0 + t) * d.dk + i] = qv * dqv - kv * dkv;
            wk[(tok0 + t) * d.dk + i] = kv * k_inter;
        }
    }
    if (!want_dg) return;
    __syncthreads();
    // reverse in-chunk running sum per feature
    for (int i = threadIdx.x; i < d.dk; i += blockDim.x) {
        float z = 0.f;
        for (int col = 0; col < d.dv; ++col) z += S[i * d.dv + col] * dS[i * d.dv + col];
        float run = expd(bval(bcum, tok0 + L - 1, dkd, i)) * z;
        for (int r = 0; r < L; ++r) run += wk[(tok0 + r) * d.dk + i];
        for (int t = L - 1; t >= 0; --t) {
            run += wq[(tok0 + t) * d.dk + i];
            if (d.kind == 3) dg[U(t) * d.dk + i] = run;
            else wq[(tok0 + t) * d.dk + i] = run;
        }
    }
    if (d.kind == 3) return;
    __syncthreads();
    for (int t = threadIdx.x; t < L; t += blockDim.x) {
        float s = 0.f;
        for (int i = 0; i < d.dk; ++i) s += wq[(tok0 + t) * d.dk + i];
        if (d.kind == 2) dg[U(t)] = s;
        else dg_tok[tok0 + t] = s;
    }
}

// dg[h] = sum_{b,t} dg_tok[b,h,t], fixed summation order (grid: H)
__global__ void k_head_reduce(Dims d, const float* __restrict__ dg_tok, float* __restrict__ dg) {
    __shared__ float part[kThreads];
    const int h = blockIdx.x;
    float s = 0.f;
    const size_t n = size_t(d.B) * d.T;
    for (size_t e = threadIdx.x; e < n; e += blockDim.x) {
        const size_t b = e / d.T, t = e % d.T;
        s += dg_tok[(b * d.H + h) * d.T + t];
    }
    part[threadIdx.x] = s;
    __syncthreads();
    for (int w = kThreads / 2; w > 0; w >>= 1) {
        if (threadIdx.x < w) part[threadIdx.x] += part[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) dg[h] = part[0];
}

struct WsFwd { bsum_t* bcum; float* states; size_t bytes; };
struct WsBwd { bsum_t* bcum; float *states, *dstates, *wq, *wk, *dg_tok; size_t bytes; };

WsFwd carve_fwd(const Dims& d, void* ws) {
    char* p = static_cast<char*>(ws);
    size_t off = 0;
    WsFwd w{};
    if (d.kind != 0) { w.bcum = reinterpret_cast<bsum_t*>(p + off); off += align256(size_t(d.BH()) * d.T * d.dkd() * sizeof(bsum_t)); }
    w.states = reinterpret_cast<float*>(p + off); off += align256(size_t(d.BH()) * d.N * d.dk * d.dv * 4);
    w.bytes = off;
    return w;
}

WsBwd carve_bwd(const Dims& d, void* ws) {
    char* p = static_cast<char*>(ws);
    size_t off = 0;
    WsBwd w{};
    const size_t st = align256(size_t(d.BH()) * d.N * d.dk * d.dv * 4);
    if (d.kind != 0) { w.bcum = reinterpret_cast<bsum_t*>(p + off); off += align256(size_t(d.BH()) * d.T * d.dkd() * sizeof(bsum_t)); }
    w.states = reinterpret_cast<float*>(p + off); off += st;
    w.dstates = reinterpret_cast<float*>(p + off); off += st;
    if (d.kind != 0) {
        w.wq = reinterpret_cast<float*>(p + off); off += align256(size_t(d.BH()) * d.T * d.dk * 4);
        w.wk = reinterpret_cast<float*>(p + off); off += align256(size_t(d.BH()) * d.T * d.dk * 4);
    }
    if (d.kind == 1) { w.dg_tok = reinterpret_cast<float*>(p + off); off += align256(size_t(d.BH()) * d.T * 4); }
    w.bytes = off;
    return w;
}

template <typename TIO>
hipError_t fwd_t(const Dims& d, const FwdArgs& a) {
    WsFwd w = carve_fwd(d, a.ws);
    const dim3 grid(d.N, d.BH()), block(kThreads);
    const int sz = d.dk * d.dv;
    auto q = static_cast<const TIO*>(a.q), k = static_cast<const TIO*>(a.k), v = static_cast<const TIO*>(a.v);
    if (d.kind != 0) { ProfScope ps(KID_GEN_CUMSUM, a.stream); hipLaunchKernelGGL(k_cumsum, grid, block, 0, a.stream, d, a.g, w.bcum); }
    { ProfScope ps(KID_GEN_STATE, a.stream); hipLaunchKernelGGL((k_local_state<TIO, 0>), grid, block, 0, a.stream, d, k, v, w.bcum, w.states); }
    { ProfScope ps(KID_GEN_SCAN, a.stream); hipLaunchKernelGGL((k_scan<false>), dim3((sz + kThreads - 1) / kThreads, d.seqs()), block, 0, a.stream, d, w.bcum,
                       w.states, a.m0, a.mT); }
    const size_t lds = size_t(d.C) * d.C * 4;
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_output<TIO>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, int(lds));
        if (e != hipSuccess) return e;
    }
    { ProfScope ps(KID_GEN_OUTPUT, a.stream); hipLaunchKernelGGL((k_output<TIO>), grid, block, lds, a.stream, d, q, k, v, w.bcum, w.states,
                       static_cast<TIO*>(a.o)); }
    return hipGetLastError();
}

template <typename TIO>
hipError_t bwd_t(const Dims& d, const BwdArgs& a) {
    WsBwd w = carve_bwd(d, a.ws);
    const dim3 grid(d.N, d.BH()), block(kThreads);
    const int sz = d.dk * d.dv;
    const dim3 sgrid((sz + kThreads - 1) / kThreads, d.seqs());
    auto q = static_cast<const TIO*>(a.q), k = static_cast<const TIO*>(a.k), v = static_cast<const TIO*>(a.v);
    auto d_o = static_cast<const TIO*>(a.d_o);
    const size_t lds = size_t(d.C) * d.C * 8;
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_grad<TIO>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, int(lds));
        if (e != hipSuccess) return e;
    }
    if (d.kind != 0) { ProfScope ps(KID_GEN_CUMSUM, a.stream); hipLaunchKernelGGL(k_cumsum, grid, block, 0, a.stream, d, a.g, w.bcum); }
    { ProfScope ps(KID_GEN_STATE, a.stream); hipLaunchKernelGGL((k_local_state<TIO, 0>), grid, block, 0, a.stream, d, k, v, w.bcum, w.states); }
    { ProfScope ps(KID_GEN_SCAN, a.stream); hipLaunchKernelGGL((k_scan<false>), sgrid, block, 0, a.stream, d, w.bcum, w.states, a.m0,
                       static_cast<float*>(nullptr)); }
    { ProfScope ps(KID_GEN_DSTATE, a.stream); hipLaunchKernelGGL((k_local_state<TIO, 1>), grid, block, 0, a.stream, d, q, d_o, w.bcum, w.dstates); }
    { ProfScope ps(KID_GEN_RSCAN, a.stream); hipLaunchKernelGGL((k_scan<true>), sgrid, block, 0, a.stream, d, w.bcum, w.dstates, a.d_mT, a.d_m0); }
    const bool want_dg = a.dg != nullptr;
    { ProfScope ps(KID_GEN_GRAD, a.stream); hipLaunchKernelGGL((k_grad<TIO>), grid, block, lds, a.stream, d, q, k, v, d_o, w.bcum, w.states, w.dstates,
                       static_cast<TIO*>(a.dq), static_cast<TIO*>(a.dk), static_cast<TIO*>(a.dv),
                       (want_dg && d.kind != 1) ? a.dg : static_cast<float*>(nullptr), w.wq, w.wk,
                       (want_dg && d.kind == 1) ? w.dg_tok : static_cast<float*>(nullptr)); }
    if (want_dg && d.kind == 1) {
        ProfScope ps(KID_HEAD_REDUCE, a.stream);
        hipLaunchKernelGGL(k_head_reduce, dim3(d.H), block, 0, a.stream, d, w.dg_tok, a.dg);
    }
    return hipGetLastError();
}

}  // namespace

namespace {
// packed input: cstart[s] = sum over earlier sequences of ceil(len / C)  (one thread; n_seq is small)
__global__ void k_chunk_starts(Dims d, int* __restrict__ cstart) {
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    int c = 0;
    cstart[0] = 0;
    for (int s = 0; s < d.nseq; ++s) {
        c += (d.cu[s + 1] - d.cu[s] + d.C - 1) / d.C;
        cstart[s + 1] = c;
    }
}
}  // namespace
hipError_t launch_chunk_starts(const Dims& d, int* cstart, hipStream_t stream) {
    hipLaunchKernelGGL(k_chunk_starts, dim3(1), dim3(64), 0, stream, d, cstart);
    return hipGetLastError();
}

size_t generic_fwd_workspace(const Dims& d) { return carve_fwd(d, nullptr).bytes; }
size_t generic_bwd_workspace(const Dims& d) { return carve_bwd(d, nullptr).bytes; }

hipError_t generic_fwd(const Dims& d, const FwdArgs& a) {
    return d.bf16 ? fwd_t<uint16_t>(d, a) : fwd_t<float>(d, a);
}
hipError_t generic_bwd(const Dims& d, const BwdArgs& a) {
    return d.bf16 ? bwd_t<uint16_t>(d, a) : bwd_t<float>(d, a);
}

}  // namespace lsm
