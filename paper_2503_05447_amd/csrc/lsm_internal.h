// Internal declarations shared by the kernels and the C-ABI front end of the
// gfx950 LSM library.  Nothing here is visible to callers.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace lsm {

// Problem geometry handed to every launcher.  N = ceil(T / C) chunks per sequence; for packed
// variable-length input (cu != NULL, B = 1) N is the total chunk count over all sequences, T the
// total token count, and no chunk straddles two sequences.
struct Dims {
    int B, H, T, dk, dv, C, N, kind;
    bool bf16;    // element type of q,k,v,o and their gradients
    int layout;   // 0: [B,H,T,d] (head-major), 1: [B,T,H,d] (token-major); same for per-token decays
    int nseq;     // packed variable-length input: number of sequences, else 0
    const int* cu;      // [nseq + 1] first token of each sequence (device memory), cu[nseq] = T
    const int* cstart;  // [nseq + 1] first chunk of each sequence (device memory, written by the library)
    bool save;    // the forward call leaves its chunk states in the workspace and the backward call reads them
    // Scalar decay kinds with d_v a multiple of 128: the value columns evolve independently, so the walkers take one
    // 128-wide slice of the value-sized tensors (v, o, d_o, dv, the value side of the states) per pass.  vm = d_v / 128
    // (value rows are vm rows of 128 elements), vs = the slice of this pass; passes after the first add to dq, dk, dg.
    int vm = 1, vs = 0;
    __host__ __device__ int BH() const { return B * H; }
    __host__ __device__ int dkd() const { return kind == 3 ? dk : 1; }  // decay values per token
    __host__ __device__ int seqs() const { return nseq ? nseq * H : B * H; }  // independent recurrences
};

// Where one chunk of one (b,h) lives.
struct ChunkPos {
    int t0, L;      // first token and number of valid tokens (L <= 0: no such chunk)
    size_t tok0;    // row of the first token in the caller's q/k/v/o arrays (rows of d_k or d_v elements)
    int ts;         // rows between consecutive tokens there
    size_t vtok0;   // the same for the value-sized arrays in units of 128 elements, at this pass's slice
    int vts;
    size_t wtok0;   // first token in the library's own per-token arrays ([BH][T] order)
    size_t slot;    // this chunk in the library's per-chunk arrays ([BH][N] order)
};
__device__ __forceinline__ ChunkPos chunk_pos_at(const Dims& d, int bh, int t0, int L, int c) {
    ChunkPos p;
    p.t0 = t0;
    p.L = L;
    p.ts = d.layout ? d.H : 1;
    p.tok0 = d.layout ? (size_t(bh / d.H) * d.T + t0) * d.H + bh % d.H : size_t(bh) * d.T + t0;
    p.vts = p.ts * d.vm;
    p.vtok0 = p.tok0 * d.vm + d.vs;
    p.wtok0 = size_t(bh) * d.T + t0;
    p.slot = size_t(bh) * d.N + c;
    return p;
}
// chunk c (grid index) of (b,h); packed input: c counts chunks over all sequences
__device__ __forceinline__ ChunkPos chunk_pos(const Dims& d, int c, int bh) {
    if (!d.cu) return chunk_pos_at(d, bh, c * d.C, min(d.C, d.T - c * d.C), c);
    int lo = 0, hi = d.nseq;  // last s with cstart[s] <= c
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (d.cstart[mid] <= c) lo = mid; else hi = mid;
    }
    if (c >= d.cstart[d.nseq]) return chunk_pos_at(d, bh, 0, 0, c);
    const int t0 = d.cu[lo] + d.C * (c - d.cstart[lo]);
    return chunk_pos_at(d, bh, t0, min(d.C, d.cu[lo + 1] - t0), c);
}
// Walk of one recurrence: q-th of Dims::seqs().  Sets the (b,h) index, the index of its edge states,
// the first chunk and the chunk count.
struct SeqWalk { int bh, edge, c0, n, tbeg, tend; };
__device__ __forceinline__ SeqWalk seq_walk(const Dims& d, int q) {
    if (!d.cu) return SeqWalk{q, q, 0, d.N, 0, d.T};
    const int s = q / d.H;
    return SeqWalk{q % d.H, q, d.cstart[s], d.cstart[s + 1] - d.cstart[s], d.cu[s], d.cu[s + 1]};
}
// k-th chunk of a walk
__device__ __forceinline__ ChunkPos walk_pos(const Dims& d, const SeqWalk& w, int k) {
    const int t0 = w.tbeg + k * d.C;
    return chunk_pos_at(d, w.bh, t0, min(d.C, w.tend - t0), w.c0 + k);
}

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

// first chunk of every sequence of a packed variable-length input: cstart[s] = sum_{s' < s} ceil(len_s' / C)
hipError_t launch_chunk_starts(const Dims& d, int* cstart, hipStream_t stream);

inline size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

// Kernel identifiers reported by the optional per-kernel timing (lsm_profile_start / _stop).
enum KernelId {
    KID_GEN_CUMSUM = 0, KID_GEN_STATE, KID_GEN_SCAN, KID_GEN_OUTPUT, KID_GEN_DSTATE, KID_GEN_RSCAN, KID_GEN_GRAD,
    KID_HEAD_REDUCE, KID_MFMA_STATE, KID_MFMA_OUTPUT, KID_MFMA_STATE_BWD, KID_MFMA_DSTATE, KID_MFMA_GRAD, KID_MFMA_PREP, KID_MFMA_VEC_PREP, KID_MFMA_VEC_DV, KID_STEP,
    KID_WALK_SUMMARY, KID_WALK_SCAN, KID_WALK_FWD, KID_WALK_GRAD, KID_DELTA_PREP, KID_DELTA_WALK, KID_DELTA_RWALK, KID_DELTA_GRAD, KID_DELTA_SUMMARY, KID_DELTA_COMBINE, KID_COUNT
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
// it runs the chunk-state scan itself and needs mfma_intra_bench_workspace() bytes
size_t mfma_intra_bench_workspace(const Dims& d);
hipError_t mfma_intra_bench(const Dims& d, const FwdArgs& a, int reps);

// Delta-rule rows (DeltaNet, Gated DeltaNet), forward: Dims::kind 0 = no decay (alpha = 1), 2 = log_alpha per token.
struct DeltaArgs {
    const void *q, *k, *v;
    const float *log_alpha, *beta, *bw, *m0;
    void* o;
    float* mT;
    void* ws;
    hipStream_t stream;
};
struct DeltaBwdArgs {
    const void *q, *k, *v;
    const float *log_alpha, *beta, *bw, *m0;
    const void* d_o;
    const float* d_mT;
    void *dq, *dk, *dv;
    float *d_log_alpha, *d_beta, *d_bw, *d_m0;
    void* ws;
    hipStream_t stream;
};
bool delta_supported(const Dims& d);
size_t delta_fwd_workspace(const Dims& d);
size_t delta_bwd_workspace(const Dims& d);
hipError_t delta_fwd(const Dims& d, const DeltaArgs& a);
hipError_t delta_bwd(const Dims& d, const DeltaBwdArgs& a);

// Recurrent single-token step (decoding): state updated in place, T of the Dims ignored.
hipError_t step(const Dims& d, const void* q, const void* k, const void* v, const float* g, float* state, void* o,
                hipStream_t stream);

// the same for the delta-rule rows; log_alpha, beta, bw: [B,H] or NULL (= 1)
hipError_t delta_step(const Dims& d, const void* q, const void* k, const void* v, const float* log_alpha, const float* beta,
                      const float* bw, float* state, void* o, hipStream_t stream);

}  // namespace lsm
