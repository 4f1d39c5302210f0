// MFMA kernel family of the chunkwise LSM path for gfx950: bf16 operands, fp32 accumulation,
// chunk = 64 tokens, d_k = 128.  This file: the chunk-state scans (the vector kind's forward and backward
// scans, the scalar kinds' reverse scan of state gradients), the per-chunk output kernel kept as the
// intra-chunk benchmark aid, and the host side; the fused chunk walkers of the scalar decay kinds
// (none / per-head / per-token scalar, d_v = 128) are in lsm_mfma_walk.h, the per-chunk kernels of the
// per-key-feature (vector) kind in lsm_mfma_vec.h (d_v = 128 or 256).
//
// Algorithm 2 of the paper generalised to a decay, per (b,h) and chunk c with chunk-local
// cumulative log-decay b_j:
//   chunk_state  U_c = sum_r e^{b_C-b_r} k_r^T v_r               (Alg. 2: M_t = K_t^T V_t)
//   scan         S_{c+1} = e^{b_C} S_c + U_c                     (Alg. 2: PrefixSum)
//   output       O = [(Q K^T) * D * Psi] V + diag(e^{b}) Q S_c   (Alg. 2: O_intra + O_inter)
// and the mirrored backward (dU_c, reverse scan, per-chunk gradients).
//
// Every contraction is a 32x32x16 bf16 MFMA.  Operand conventions (wave64, l = lane, half = l/32):
//   A operand: lane holds A[m = l%32][k = 8*half + e],  e = 0..7
//   B operand: lane holds B[k = 8*half + e][n = l%32]
//   D result : lane holds D[m = 8*g + 4*half + j][n = l%32] in register 4*g + j
// Tiles arrive feature-contiguous ([token][feature] rows).  A contraction over FEATURES reads its
// operands as 16-byte row pieces (frag).  A contraction over TOKENS reads them with the LDS transpose
// read (frag_tr: lane = feature, 8 tokens), which needs no transposed copy.  Rounded products (scores,
// decayed operands, states where it matters) are carried as a bf16 head plus a bf16 remainder and
// cost two MFMAs.
#include "lsm_mfma_dev.h"

#include <atomic>
#include <mutex>
#include <vector>

namespace lsm {
namespace {


// Log-decay of this lane's token (every wave loads, only wave 0's value is used).  To be called
// BEFORE the kernel's other global loads: loads return in order, so waiting for this one later
// leaves the younger ones in flight, whereas as the youngest it would drain the whole queue.
__device__ __forceinline__ float decay_gload(const Dims& d, const float* g, int bh, const ChunkPos& cp, int lane) {
    if (d.kind == 0) return 0.f;
    return g[d.kind == 1 ? size_t(bh % d.H) : cp.tok0 + size_t(min(lane, cp.L - 1)) * cp.ts];
}
// Chunk-local inclusive cumulative log-decay b_j, j = 0..63, into LDS (tokens >= L carry g = 0) from
// the values of decay_gload.  Called by all threads; only wave 0 works.  Caller synchronises afterwards.
__device__ __forceinline__ void cumulative_decay(float gval, int L, float* bs, int tid) {
    if (tid >= 64) return;
    float x = tid < L ? gval : 0.f;
    for (int off = 1; off < 64; off <<= 1) {
        const float y = __shfl_up(x, off, 64);
        if (tid >= off) x += y;
    }
    bs[tid] = x;
}

// ---------------------------------------------------------------------------------------------
// Decay preparation for the state passes: per chunk c of (b,h), padded to 64 tokens,
//   wdec[t] = e^{b_C - b_t} ,  winc[t] = e^{b_t} ,  lam[c] = e^{b_C}
// (grid: N x BH, one wave).  Keeps the wave scan and the exponentials out of the sequential loop.
__global__ __launch_bounds__(64) void mk_decay_prep(Dims d, const float* __restrict__ g, float* __restrict__ wdec,
                                                    float* __restrict__ winc, float* __restrict__ lam) {
    const int c = blockIdx.x, bh = blockIdx.y, lane = threadIdx.x;
    const ChunkPos cp = chunk_pos(d, c, bh);
    const int L = cp.L;
    if (L <= 0) return;
    float x = 0.f;
    if (lane < L) x = d.kind == 1 ? g[bh % d.H] : g[cp.tok0 + size_t(lane) * cp.ts];
    for (int off = 1; off < 64; off <<= 1) {
        const float y = __shfl_up(x, off, 64);
        if (lane >= off) x += y;
    }
    const float bC = __shfl(x, 63, 64);
    const size_t base = cp.slot * C;
    wdec[base + lane] = __expf(bC - x);
    winc[base + lane] = __expf(x);
    if (lane == 0) lam[cp.slot] = __expf(bC);
}

// ---------------------------------------------------------------------------------------------
// Chunk states and the scan over chunks, fused: one wave owns a 32 x 32 block of the d_k x d_v
// state in MFMA accumulators (fp32) and walks the chunks of its sequence in order,
//     S_{c+1} = e^{b_C} S_c + sum_r (k_r e^{b_C - b_r})^T v_r ,
// writing the bf16 copy of S_c that the per-chunk kernels consume before each update.
//   MODE 0: forward states, stored S^T [v][i]   (A side = k decayed, B side = v)
//   MODE 1: backward recomputation, stored S [i][v]   (A side = v, B side = k decayed)
//   MODE 2: reverse scan of state gradients, stored dS [i][v]: slot c receives the gradient of the
//           state at the END of chunk c;  dS_c = e^{b_C} dS_{c+1} + sum_j d_o_j^T (q_j e^{b_j})
//           (A side = d_o, B side = q decayed)
// Both operands of the token contraction come from identity turns, so their k order agrees.  The
// decayed operand is split into a bf16 head and a bf16 remainder (two MFMAs) so that the rounding of
// k * w does not show in a state that one token dominates.  DEC = false (no decay) skips all of it.
// The loop is software-pipelined: global loads run three chunks ahead in rotating register sets, the
// tiles of the next two chunks sit in LDS (weighted and split on the way in) while this one is contracted.
// edge_in = M_0 (or d M_T), edge_out = M_T (or d M_0), fp32 [i][v], either may be NULL.
// states_rem (may be NULL) receives the remainder S - bf16(S) in the same layout as 8-bit floats: the decay
// gradient contracts q_u S d_o_u^T into one scalar per token, where the 2^-9 rounding of a state that
// a single token dominates is visible.
constexpr int LDB = 40;  // row stride (elements) of a 64 x 32 B-side slice in LDS
// LDS: 2 x (A tile 64 x LD | B slice head 64 x LDB | B slice remainder 64 x LDB) for chunks k+1, k+2
//      | one 32 x LD stage for the scans that also store a block untransposed (the transposed order
//        leaves straight from the registers, see state_store_direct)
constexpr int kStateTile = C * LD + 2 * C * LDB;
constexpr int kStateLdsNone = 2 * kStateTile * 2;                  // transposed stores only
constexpr int kStateLdsPlain = (2 * kStateTile + 32 * LD) * 2;     // with the stage of an untransposed copy

struct StateRegs {  // one thread's share of a chunk on its way from global memory to LDS
    u32x4 a[4], b, blo;  // blo: remainder plane of the B slice (vector decay: both planes arrive precomputed)
    float w;             // weight of the B-slice row this thread carries
    float lam;           // e^{b_C}: one per chunk, or (vector decay) the one of this lane's state column
    int L;               // valid tokens of the chunk; rows beyond are zeroed on the way to LDS
};

struct StateArgs {
    const uint16_t *xa, *xb;
    const float *wts, *lam;
    uint16_t *states, *states_rem;
    const float* edge_in;
    float* edge_out;
    // vector decay only
    const uint16_t* xb_lo;  // remainder plane of the decayed B-side operand
    int a_stride;           // row stride (elements) of the A-side operand = d_v
    int vh_count;           // 128-wide value slices per (b,h); each is scanned as a sequence of its own
    uint16_t* states_twin;  // MODE 2 only: second copy of the head, untransposed (dS^T [v][i]), or NULL
    // scan cut into segments (seg_n > 1; grid = seg_n times the plain one): segment s walks chunks
    // [s seg_m, (s+1) seg_m) from the state in seg_bound, which holds fp32 [i][v] entry states at a finer grain
    // (one per fine_m chunks, fine_n slots per sequence, slot f = the state the walk enters fine segment f with)
    const float* seg_bound;
    int seg_m, seg_n, fine_m, fine_n;
};

// coalesced: the A side as whole 256-byte rows (16 lanes per row), the B side as 64-byte row slices.
// Branch-free (rows beyond the ragged end are read from the last valid row and zeroed afterwards) so
// that the compiler can count outstanding loads exactly and need not drain the queue.
template <bool DEC, bool VEC>
__device__ __forceinline__ void state_gload(const Dims& d, const uint16_t* xa, const uint16_t* xb,
                                            const uint16_t* xb_lo, const float* wts, const float* lam, int a_stride,
                                            const ChunkPos& cp, size_t lamslot, int fb0, int tid, StateRegs& r) {
    const int L = cp.L;
    const int astride = VEC ? a_stride : D * d.vm;  // scalar kinds: the A side is value-sized (d_o), one 128-wide slice per pass
    // The set of this chunk carries e^{b_C} of chunk `lamslot`, the one that is being accumulated when
    // this set goes to LDS: the factor is then read from a set that has arrived, and no loaded value is
    // copied from iteration to iteration (such a copy waits for every load in flight).
    if (VEC) {
        r.lam = lam[lamslot * D + fb0 + (tid & 31)];
    } else if (DEC) {
        r.w = wts[cp.slot * C + (tid >> 2)];
        r.lam = lam[lamslot];
    }
    _Pragma("unroll") for (int it = 0; it < 4; ++it) {
        const int p = tid + kThreads * it, row = p >> 4, cpp = p & 15;
        r.a[it] = *reinterpret_cast<const u32x4*>(xa + (cp.tok0 + size_t(min(row, L - 1)) * cp.ts) * astride + cpp * 8);
    }
    // nothing is computed on the loaded values here (the ragged tail is zeroed when they go to LDS): an
    // ALU operation at this point would make the wave wait for the load it has just issued
    r.L = L;
    const int row = min(tid >> 2, L - 1), cpp = tid & 3;
    // vector decay: the decayed operand comes from the library's own planes ([BH*T][128] order)
    const size_t boff = (VEC ? cp.wtok0 + row : cp.tok0 + size_t(row) * cp.ts) * D + fb0 + cpp * 8;
    r.b = *reinterpret_cast<const u32x4*>(xb + boff);
    if (VEC) r.blo = *reinterpret_cast<const u32x4*>(xb_lo + boff);
}
// The B slice carries the decay: each row is multiplied by its token's weight in fp32 and stored as a
// bf16 head plus a bf16 remainder, once per workgroup.
template <bool DEC, bool VEC>
__device__ __forceinline__ void state_to_lds(const StateRegs& r, uint16_t* bufA, uint16_t* bufB, int tid) {
    _Pragma("unroll") for (int it = 0; it < 4; ++it) {
        const int p = tid + kThreads * it, row = p >> 4, cp = p & 15;
        const uint32_t keep = row < r.L ? 0xffffffffu : 0u;
        *reinterpret_cast<u32x4*>(bufA + row * LD + cp * 8) =
            u32x4{r.a[it].x & keep, r.a[it].y & keep, r.a[it].z & keep, r.a[it].w & keep};
    }
    uint16_t* dst = bufB + (tid >> 2) * LDB + (tid & 3) * 8;
    const uint32_t keep = (tid >> 2) < r.L ? 0xffffffffu : 0u;
    const u32x4 rb = {r.b.x & keep, r.b.y & keep, r.b.z & keep, r.b.w & keep};
    if (VEC) {
        *reinterpret_cast<u32x4*>(dst) = rb;
        *reinterpret_cast<u32x4*>(dst + C * LDB) = u32x4{r.blo.x & keep, r.blo.y & keep, r.blo.z & keep, r.blo.w & keep};
    } else if (DEC) {
        u32x4 hi, lo;
        _Pragma("unroll") for (int p = 0; p < 4; ++p) {
            const float x0 = bf16_lo(rb[p]) * r.w, x1 = bf16_hi(rb[p]) * r.w;
            const uint32_t h = pack2(x0, x1);
            hi[p] = h;
            lo[p] = pack2(x0 - bf16_lo(h), x1 - bf16_hi(h));
        }
        *reinterpret_cast<u32x4*>(dst) = hi;
        *reinterpret_cast<u32x4*>(dst + C * LDB) = lo;
    } else {
        *reinterpret_cast<u32x4*>(dst) = rb;
    }
}

// Chunk states live in HBM "fragment-major": the 128 x 128 matrix X whose rows are the m index and
// whose columns are the contraction index of the consumer's MFMA is stored as
//     [row / 32][col / 16][(col / 8) % 2][row % 32][col % 8] ,
// so that the A operand of k-step ks for the 32 rows of block w is one contiguous KiB with lane l
// at byte 16 l: the per-chunk kernels read it with fully coalesced loads, and the scan writes
// 512-byte runs.
__device__ __forceinline__ size_t state_frag_off(int blk, int ks, int lane) {
    return (size_t(blk * 8 + ks) * 64 + lane) * 8;
}
// One wave's staged 32 x 32 block -> global memory.  Stage row r = row r of the stored block `rowblk`,
// stage columns 32 mb .. +31 = its columns 32 colblk .. +31.  The wave reads back only what it staged
// itself, and LDS serves a wave's accesses in order: no barrier.
template <bool STREAM = true>
__device__ __forceinline__ void state_store(uint16_t* dst, const uint16_t* stage, int mb, int rowblk, int colblk,
                                            int lane) {
    _Pragma("unroll") for (int it = 0; it < 2; ++it) {
        const int piece = 2 * it + (lane >> 5), ksl = piece >> 1, hf = piece & 1, r = lane & 31;
        const u32x4 val = *reinterpret_cast<const u32x4*>(stage + r * LD + 32 * mb + 16 * ksl + 8 * hf);
        u32x4* p = reinterpret_cast<u32x4*>(dst + state_frag_off(rowblk, 2 * colblk + ksl, 32 * hf + r));
        // written once, read by a later kernel: keep it from displacing the shared input tiles in L2
        if (STREAM) __builtin_nontemporal_store(val, p);
        else *p = val;
    }
}

// The same block -> global memory without LDS, for the transposed order (stored row = the lane's column
// n, stored columns = the block's rows m).  In D layout lanes l and l + 32 hold complementary halves
// (4 + 4 rows) of every group of 8 rows; one v_permlane32_swap per dword hands each lane a whole group:
// the lower lanes the even groups, the upper lanes the odd ones, i.e. exactly the 16 bytes that lane
// 32 hf + n of fragment (rowblk, 2 mb + q) holds, and a wave stores one contiguous KiB per instruction.
__device__ __forceinline__ void state_store_direct(uint16_t* dst, int rowblk, int mb, int lane, const f32x16& acc) {
    _Pragma("unroll") for (int q = 0; q < 2; ++q) {
        const uint32_t a0 = pack2(acc[8 * q + 0], acc[8 * q + 1]), a1 = pack2(acc[8 * q + 2], acc[8 * q + 3]);
        const uint32_t b0 = pack2(acc[8 * q + 4], acc[8 * q + 5]), b1 = pack2(acc[8 * q + 6], acc[8 * q + 7]);
        const auto s0 = __builtin_amdgcn_permlane32_swap(a0, b0, false, false);
        const auto s1 = __builtin_amdgcn_permlane32_swap(a1, b1, false, false);
        const u32x4 val = {s0[0], s1[0], s0[1], s1[1]};
        __builtin_nontemporal_store(val, reinterpret_cast<u32x4*>(dst + state_frag_off(rowblk, 2 * mb + q, lane)));
    }
}
// with the 8-bit remainder plane: (x - head) * 2^8 as an 8-bit float, same element order, one byte each
__device__ __forceinline__ void state_store_direct_split8(uint16_t* dst, uint8_t* dst8, int rowblk, int mb, int lane,
                                                          const f32x16& acc) {
    _Pragma("unroll") for (int q = 0; q < 2; ++q) {
        uint32_t h[4];
        int r8[2];
        _Pragma("unroll") for (int gg = 0; gg < 2; ++gg) {
            const int x = 8 * q + 4 * gg;
            h[2 * gg] = pack2(acc[x], acc[x + 1]);
            h[2 * gg + 1] = pack2(acc[x + 2], acc[x + 3]);
            int v = __builtin_amdgcn_cvt_pk_bf8_f32((acc[x] - bf16_lo(h[2 * gg])) * kRem8Scale,
                                                    (acc[x + 1] - bf16_hi(h[2 * gg])) * kRem8Scale, 0, false);
            r8[gg] = __builtin_amdgcn_cvt_pk_bf8_f32((acc[x + 2] - bf16_lo(h[2 * gg + 1])) * kRem8Scale,
                                                     (acc[x + 3] - bf16_hi(h[2 * gg + 1])) * kRem8Scale, v, true);
        }
        const auto s0 = __builtin_amdgcn_permlane32_swap(h[0], h[2], false, false);
        const auto s1 = __builtin_amdgcn_permlane32_swap(h[1], h[3], false, false);
        const auto sr = __builtin_amdgcn_permlane32_swap(uint32_t(r8[0]), uint32_t(r8[1]), false, false);
        const size_t off = state_frag_off(rowblk, 2 * mb + q, lane);
        __builtin_nontemporal_store(u32x4{s0[0], s1[0], s0[1], s1[1]}, reinterpret_cast<u32x4*>(dst + off));
        __builtin_nontemporal_store(u32x2{sr[0], sr[1]}, reinterpret_cast<u32x2*>(dst8 + off));
    }
}

// VEC (per-key-feature decay): the decayed operand (k e^{b_C-b} or q e^{b}) arrives precomputed as a
// head and a remainder plane and is always the B side, so that a state column n is one key feature i
// and e^{b_C[i]} is one factor per lane; the A side is a 128-wide slice of the value-sized operand
// (row stride d_v), each slice being scanned like a sequence of its own.
//   MODE 3 (VEC only): forward states with the operands of MODE 1, stored S^T [v][i] like MODE 0.
//   MODE 2 with VEC: states_twin, when given, receives a second copy dS^T [v][i] (for the dv kernel).
//   SAVE (MODE 3 only): the forward scan also leaves what the backward pass needs of it, the states in
//   the order MODE 1 stores them (S [i][v], into states_twin) and their 8-bit remainder plane (states_rem).
template <int MODE, bool DEC, bool REM, bool VEC, bool SAVE = false>
__device__ __forceinline__ void state_scan_body(const Dims& d, const StateArgs& sa, int wg_id, int wg_count,
                                                unsigned char* smem) {
    const uint16_t* __restrict__ xa = sa.xa;
    const uint16_t* __restrict__ xb = sa.xb;
    const uint16_t* __restrict__ xb_lo = sa.xb_lo;
    const float* __restrict__ wts = sa.wts;
    const float* __restrict__ lam = sa.lam;
    uint16_t* __restrict__ states = sa.states;
    uint16_t* __restrict__ states_rem = sa.states_rem;
    uint16_t* __restrict__ states_twin = sa.states_twin;
    const float* __restrict__ edge_in = sa.edge_in;
    float* __restrict__ edge_out = sa.edge_out;
    uint16_t* tiles = reinterpret_cast<uint16_t*>(smem);         // [2][kStateTile]
    uint16_t* stage = tiles + 2 * kStateTile;                    // [32 * LD]: the untransposed copy, if any
    // The four workgroups of a sequence read the same A-side rows.  Workgroups are dealt to the 8
    // XCDs round-robin by linear id, so the id is decoded such that those four share an XCD (and
    // its L2): id = xcd + 8 * (4 * (seq / 8) + nb), seq = xcd + 8 * (seq / 8).
    int nb, seq;
    const int nsegs = sa.seg_n > 1 ? sa.seg_n : 1, seg = wg_id / (wg_count / nsegs);
    {
        const int nwg = wg_count / nsegs, id = wg_id % nwg, full = (nwg / 32) * 32;  // 32 = 8 XCDs x 4 blocks
        if (id < full) {
            const int xcd = id & 7, slot = id >> 3;
            nb = slot & 3;
            seq = xcd + 8 * (slot >> 2);
        } else {  // tail when the number of sequences is not a multiple of 8
            nb = (id - full) & 3;
            seq = (full >> 2) + ((id - full) >> 2);
        }
    }
    const int vh = VEC ? seq % sa.vh_count : 0, nvh = VEC ? sa.vh_count : 1;
    const SeqWalk walk = seq_walk(d, VEC ? seq / sa.vh_count : seq);
    const int kbeg = nsegs > 1 ? seg * sa.seg_m : 0, kend = nsegs > 1 ? min(walk.n, kbeg + sa.seg_m) : walk.n;
    if (seg > 0 && kend <= kbeg) return;  // a sequence shorter than this segment's start
    const int cnt = kend - kbeg;  // chunks to walk
    const int tid = threadIdx.x, lane = tid & 63, mb = tid >> 6;
    const int n = lane & 31, half = lane >> 5;
    constexpr int sz = D * D;
    const int erow = VEC ? sa.a_stride : D * d.vm;  // row stride of the fp32 edge states [i][v]
    const int vcol = VEC ? D * vh : D * d.vs;       // first value column of this scan in the value-sized arrays

    // acc[4g+j] = state element (m = 32mb + 8g + 4half + j, n = 32nb + lane%32); MODE 0: m = i, else m = v
    f32x16 acc = {0};
    if (nsegs > 1) {
        // MODE 2 walks backward: it enters with the state of the last fine segment it covers
        const int nfine = max(1, (walk.n + sa.fine_m - 1) / sa.fine_m), per = sa.seg_m / sa.fine_m;
        const int f = MODE == 2 ? min(nfine, (seg + 1) * per) - 1 : seg * per;
        const float* e = sa.seg_bound + (size_t(seq) * sa.fine_n + f) * D * D;
        _Pragma("unroll") for (int r = 0; r < 16; ++r) {
            const int mm = 32 * mb + 8 * (r >> 2) + 4 * half + (r & 3), nn = 32 * nb + n;
            acc[r] = MODE == 0 ? e[mm * D + nn] : e[nn * D + mm];
        }
    } else if (edge_in) {
        const float* e = edge_in + size_t(walk.edge) * D * erow + vcol;
        _Pragma("unroll") for (int r = 0; r < 16; ++r) {
            const int mm = 32 * mb + 8 * (r >> 2) + 4 * half + (r & 3), nn = 32 * nb + n;
            acc[r] = MODE == 0 ? e[mm * erow + nn] : e[nn * erow + mm];
        }
    }
    const int first = MODE == 2 ? kend - 1 : kbeg, step = MODE == 2 ? -1 : 1;
    // the state this walk ends with leaves through edge_out only where the walk ends the sequence
    if (nsegs > 1 && (MODE == 2 ? seg != 0 : kend < walk.n)) edge_out = nullptr;
    auto bufA = [&](int k) { return tiles + (k & 1) * kStateTile; };
    auto bufB = [&](int k) { return tiles + (k & 1) * kStateTile + C * LD; };
    auto slot = [&](int k) { return ((size_t(walk.bh) * d.N + walk.c0 + (first + step * k)) * nvh + vh) * sz; };
    const uint16_t* xav = xa + vcol;
    auto gload = [&](int kc, StateRegs& r) {
        // the kc-th chunk of the walk (clamped at the end); it goes to LDS during iteration kc - 2
        const int c = first + step * min(kc, cnt - 1), clam = first + step * min(max(kc - 2, 0), cnt - 1);
        state_gload<DEC, VEC>(d, xav, xb, xb_lo, wts, lam, sa.a_stride, walk_pos(d, walk, c),
                              size_t(walk.bh) * d.N + walk.c0 + clam, 32 * nb, tid, r);
    };

    // prologue: chunks 0 and 1 -> LDS, chunk 2 in flight.  Global loads are issued two iterations
    // before their data is written to LDS: one iteration is shorter than a trip to HBM.
    StateRegs r0, r1, r2;
    if (cnt <= 0) {  // an empty sequence of a packed input: the state passes through
        if (edge_out) {
            float* e = edge_out + size_t(walk.edge) * D * erow + vcol;
            _Pragma("unroll") for (int x = 0; x < 16; ++x) {
                const int mm = 32 * mb + 8 * (x >> 2) + 4 * half + (x & 3), nn = 32 * nb + n;
                if (MODE == 0) e[mm * erow + nn] = acc[x];
                else e[nn * erow + mm] = acc[x];
            }
        }
        return;
    }
    gload(0, r0);
    if (cnt > 1) gload(1, r1);
    state_to_lds<DEC, VEC>(r0, bufA(0), bufB(0), tid);
    if (cnt > 1) {
        state_to_lds<DEC, VEC>(r1, bufA(1), bufB(1), tid);
    }
    gload(2, r0);
    gload(3, r1);
    __syncthreads();

    // One chunk, straight-line code: rw holds chunk k+2 (loaded three iterations ago, written to LDS
    // at the end), rl receives chunk k+4; chunk indices past the end are clamped (the data lands in a
    // buffer nobody reads).  The three register sets rotate by unrolling, never by copying: a copy
    // would wait for the load issued in the same iteration.
    auto iteration = [&](int k, StateRegs& rw, StateRegs& rl) {
        gload(k + 4, rl);
        // stage the state this chunk starts from (MODE 2: the gradient this chunk ends with)
        uint16_t* sh = stage;
        constexpr bool kTwin = VEC && MODE == 2;  // second copy, untransposed
        if (MODE == 3 || (kTwin && states_twin)) {
            _Pragma("unroll") for (int x = 0; x < 16; ++x)
                sh[(8 * (x >> 2) + 4 * half + (x & 3)) * LD + 32 * mb + n] = uint16_t(pack2(acc[x], 0.f));
        }
        // the transposed order needs no staging: registers -> global memory
        if (MODE != 3 || SAVE) {
            uint16_t* tdst = (MODE == 3 ? states_twin : states) + slot(k);
            if (states_rem) state_store_direct_split8(tdst, reinterpret_cast<uint8_t*>(states_rem) + slot(k), nb, mb, lane, acc);
            else state_store_direct(tdst, nb, mb, lane, acc);
        }
        if (DEC) {
            const float lam_cur = rw.lam;
            _Pragma("unroll") for (int x = 0; x < 16; ++x) acc[x] *= lam_cur;
        }
        // acc[m][n] += sum_t A[t][32mb + m] * Bw[t][n]: both operands read token-major out of LDS
        const uint16_t *ta = bufA(k), *tb = bufB(k);
        _Pragma("unroll") for (int ks = 0; ks < 4; ++ks) {
            const bf16x8 fa = frag_tr(ta, LD, 16 * ks, 32 * mb, lane);
            acc = mfma(fa, frag_tr(tb, LDB, 16 * ks, 0, lane), acc);
            if (DEC) acc = mfma(fa, frag_tr(tb + C * LDB, LDB, 16 * ks, 0, lane), acc);
        }
        __syncthreads();  // every wave is done with the tiles of chunk k
        state_to_lds<DEC, VEC>(rw, bufA(k), bufB(k), tid);  // chunk k+2; read again two barriers from now
        // the untransposed copy: stage row = state row m (block mb), stage columns = state columns (block nb)
        if (MODE == 3) state_store<false>(states + slot(k), sh, mb, mb, nb, lane);
        if (kTwin && states_twin) state_store(states_twin + slot(k), sh, mb, mb, nb, lane);
    };
    int k = 0;
    for (; k + 2 < cnt; k += 3) {
        iteration(k, r0, r2);
        iteration(k + 1, r1, r0);
        iteration(k + 2, r2, r1);
    }
    if (k < cnt) iteration(k, r0, r2);
    if (k + 1 < cnt) iteration(k + 1, r1, r0);
    __syncthreads();
    if (edge_out) {
        float* e = edge_out + size_t(walk.edge) * D * erow + vcol;
        _Pragma("unroll") for (int x = 0; x < 16; ++x) {
            const int mm = 32 * mb + 8 * (x >> 2) + 4 * half + (x & 3), nn = 32 * nb + n;
            if (MODE == 0) e[mm * erow + nn] = acc[x];
            else e[nn * erow + mm] = acc[x];
        }
    }
}

template <int MODE, bool DEC, bool SAVE = false>
__global__ __launch_bounds__(kThreads) void mk_state_seq(Dims d, StateArgs sa) {
    extern __shared__ __align__(16) unsigned char smem[];
    state_scan_body<MODE, DEC, false, false, SAVE>(d, sa, blockIdx.x, gridDim.x, smem);
}


// D[m][n] = sum_f Am[m0 + m][f] * Bm[n0 + n][f] over the 128 features of two row-major LDS tiles
__device__ __forceinline__ f32x16 score_block(const uint16_t* Am, int m0, const uint16_t* Bm, int n0, int n, int half) {
    // all sixteen fragments are requested before the first MFMA so that one LDS latency is paid, not eight
    bf16x8 fa[8], fb[8];
    _Pragma("unroll") for (int ks = 0; ks < 8; ++ks) {
        fa[ks] = frag(Am, LD, m0 + n, 16 * ks + 8 * half);
        fb[ks] = frag(Bm, LD, n0 + n, 16 * ks + 8 * half);
    }
    __builtin_amdgcn_sched_barrier(0);  // keep the requests above, the MFMAs below
    f32x16 acc = {0};
    _Pragma("unroll") for (int ks = 0; ks < 8; ++ks) acc = mfma(fa[ks], fb[ks], acc);
    return acc;
}

// mask and decay of a score block in D layout; ROWS_R: rows index keys r and the lane's column a query j
template <bool ROWS_R>
__device__ __forceinline__ void decay_mask(f32x16& acc, int m0, int ncol, const float* bs, int half) {
    const float bn = bs[ncol];
    _Pragma("unroll") for (int g = 0; g < 4; ++g) {
        const float4 bm = *reinterpret_cast<const float4*>(bs + m0 + 8 * g + 4 * half);
        const float bmv[4] = {bm.x, bm.y, bm.z, bm.w};
        _Pragma("unroll") for (int jj = 0; jj < 4; ++jj) {
            const int mi = m0 + 8 * g + 4 * half + jj, x = 4 * g + jj;
            const int j = ROWS_R ? ncol : mi, r = ROWS_R ? mi : ncol;
            const float e = ROWS_R ? bn - bmv[jj] : bmv[jj] - bn;
            acc[x] = r <= j ? acc[x] * __expf(e) : 0.f;
        }
    }
}

// sum over this lane's 16 features of x[tok][32w + ...] * acc[...]
__device__ __forceinline__ float row_dot(const uint16_t* X, int tok, int wave, int half, const f32x16& a) {
    float s = 0.f;
    _Pragma("unroll") for (int gg = 0; gg < 4; ++gg) {
        const u32x2 x = *reinterpret_cast<const u32x2*>(X + tok * LD + 32 * wave + 8 * gg + 4 * half);
        s += bf16_lo(x.x) * a[4 * gg] + bf16_hi(x.x) * a[4 * gg + 1] + bf16_lo(x.y) * a[4 * gg + 2] +
             bf16_hi(x.y) * a[4 * gg + 3];
    }
    return s;
}

// ---------------------------------------------------------------------------------------------
// Output of one chunk:  O^T[v][j] = e^{b_j} sum_i S^T[v][i] q_j[i] + sum_{r<=j} V^T[v][r] P[j][r],
// P[j][r] = (q_j . k_r) e^{b_j - b_r}.   Wave w owns v in [32w, 32w+32): the inter part with the state
// rows as A operand straight from global memory, then the intra part with V^T from the LDS transpose
// read.  Each of the three 32 x 32 blocks of P is computed by ONE wave (mask and decay on its
// accumulators) and handed to the others through LDS as a bf16 head plus a bf16 remainder (an output
// that one key dominates would otherwise carry the full 2^-9 rounding of its score); the head goes
// over the Q tile and the remainder over the K tile, both dead by then, so the kernel stays at 52 KiB
// of LDS.
// LDS: Q | K (later the O stage) | V (64 x LD each) | bs
// REPEAT (benchmark aid): the compute phase runs `reps` times on the tiles resident in LDS, so that
// the rate of the intra-chunk arithmetic can be measured without the HBM traffic that bounds the
// streamed kernel; the stored result is that of the last pass, identical to reps = 1.
// The V tile is only ever read through the transpose read, whose 16-lane groups fetch 4 rows x 32 bytes: with the row
// stride of the other tiles (68 words, == 4 mod 64: conflict-free for 16-byte row reads) consecutive rows overlap in
// half of their banks; 80 words (== 16 mod 64) lets the 4 rows x 2 groups of a half-wave tile the 64 banks exactly.
constexpr int LDV = D + 32;
constexpr int kOutLds = 2 * C * LD * 2 + C * LDV * 2 + C * 4;
constexpr int kOutLdsRepeat = kOutLds + 2 * C * LDP * 2;

template <bool REPEAT>
__global__ __launch_bounds__(kThreads, 3) void mk_output(Dims d, const uint16_t* __restrict__ q,
                                                         const uint16_t* __restrict__ k,
                                                         const uint16_t* __restrict__ v, const float* __restrict__ g,
                                                         const uint16_t* __restrict__ states,
                                                         uint16_t* __restrict__ o, int reps) {
    extern __shared__ __align__(16) unsigned char smem[];
    uint16_t* Q = reinterpret_cast<uint16_t*>(smem);
    uint16_t* K = Q + C * LD;
    uint16_t* V = K + C * LD;
    float* bs = reinterpret_cast<float*>(V + C * LDV);
    uint16_t* stage = K;

    const int c = blockIdx.x, bh = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const ChunkPos cp = chunk_pos(d, c, bh);
    const int L = cp.L;
    if (L <= 0) return;  // packed input: the grid is sized for an upper bound of the chunk count
    const size_t tok0 = cp.tok0;
    const int ts = cp.ts;
    const int n = lane & 31, half = lane >> 5;

    // decay first, then the tiles, the state rows after them (loads return in order; the rows are
    // needed only by the MFMAs)
    const float gval = decay_gload(d, g, bh, cp, lane);
    TileRegs tq, tk, tv;
    tile_gload(tq, q, tok0, ts, L, tid);
    tile_gload(tk, k, tok0, ts, L, tid);
    tile_gload(tv, v, tok0, ts, L, tid);
    // state rows of this wave straight from global memory: A operand [m = v][k = i]
    const uint16_t* St = states + cp.slot * D * D;
    bf16x8 sfrag[8];
    _Pragma("unroll") for (int ks = 0; ks < 8; ++ks)
        sfrag[ks] = __builtin_nontemporal_load(reinterpret_cast<const bf16x8*>(St + state_frag_off(wave, ks, lane)));

    tile_commit(Q, tq, L, tid);
    tile_commit(K, tk, L, tid);
    _Pragma("unroll") for (int it = 0; it < 4; ++it) {  // tile_commit with the V tile's own row stride
        const int p = tid + kThreads * it, row = p >> 4, cpp = p & 15;
        const uint32_t keep = row < L ? 0xffffffffu : 0u;
        *reinterpret_cast<u32x4*>(V + row * LDV + cpp * 8) = u32x4{tv.v[it].x & keep, tv.v[it].y & keep, tv.v[it].z & keep, tv.v[it].w & keep};
    }
    cumulative_decay(gval, L, bs, tid);
    __syncthreads();

    PackedBlock res[2];
    // each of the three score blocks is computed by one wave and handed to the others through LDS (head
    // over the Q tile, remainder over the K tile, both dead by then; the repeat variant, which needs Q
    // and K again, has room of its own behind bs)
    uint16_t* Ph = REPEAT ? reinterpret_cast<uint16_t*>(bs + C) : Q;
    uint16_t* Pl = REPEAT ? Ph + C * LDP : K;
    for (int rep = 0; rep < (REPEAT ? reps : 1); ++rep) {
        if (REPEAT) asm volatile("" ::: "memory");  // the tiles are read again in every pass
        f32x16 acc[2], P = {0};
        _Pragma("unroll") for (int jb = 0; jb < 2; ++jb) {
            const int j = 32 * jb + n;
            acc[jb] = f32x16{0};
            _Pragma("unroll") for (int ks = 0; ks < 8; ++ks)
                acc[jb] = mfma(sfrag[ks], frag(Q, LD, j, 16 * ks + 8 * half), acc[jb]);
            const float w = __expf(bs[j]);
            _Pragma("unroll") for (int x = 0; x < 16; ++x) acc[jb][x] *= w;
        }
        const int pjb = wave ? 1 : 0, prb = wave == 2 ? 1 : 0;  // wave 0: (0,0), wave 1: (1,0), wave 2: (1,1)
        if (wave < 3) {
            P = score_block(K, 32 * prb, Q, 32 * pjb, n, half);  // D[m = r][n = j] = k_r . q_j
            decay_mask<true>(P, 32 * prb, 32 * pjb + n, bs, half);
        }
        __syncthreads();  // every wave is done with Q and K (and, in a repeated pass, with the previous P)
        if (wave < 3) store_block_t_split(Ph, Pl, LDP, 32 * pjb + n, 32 * prb, half, P);
        __syncthreads();
        _Pragma("unroll") for (int jb = 0; jb < 2; ++jb) {
            const int j = 32 * jb + n;
            _Pragma("unroll") for (int ks = 0; ks < 2 * (jb + 1); ++ks) {  // keys r >= 32 never reach queries j < 32
                const bf16x8 vt = frag_tr(V, LDV, 16 * ks, 32 * wave, lane);
                acc[jb] = mfma(vt, frag(Ph, LDP, j, 16 * ks + 8 * half), acc[jb]);
                acc[jb] = mfma(vt, frag(Pl, LDP, j, 16 * ks + 8 * half), acc[jb]);
            }
            res[jb] = pack_block(acc[jb]);
        }
    }
    __syncthreads();  // every wave is done with the score tiles
    _Pragma("unroll") for (int jb = 0; jb < 2; ++jb) store_packed(stage, LD, 32 * jb + n, 32 * wave, half, res[jb]);
    __syncthreads();
    store_tile(o, stage, tok0, ts, L, tid);
}

// dg[h] = sum over batch elements and chunks of the per-chunk sums dg_chunk[b,h,c], in a fixed order (grid: H)
__global__ void mk_head_reduce(Dims d, const float* __restrict__ dg_tok, float* __restrict__ dg) {
    __shared__ float part[kThreads];
    const int h = blockIdx.x;
    float s = 0.f;
    const int nc = d.cu ? d.cstart[d.nseq] : d.N;  // packed input: d.N is an upper bound, the rest was never written
    const size_t nn = size_t(d.B) * nc;
    for (size_t e = threadIdx.x; e < nn; e += blockDim.x) s += dg_tok[((e / nc) * d.H + h) * d.N + e % nc];
    part[threadIdx.x] = s;
    __syncthreads();
    for (int w = kThreads / 2; w > 0; w >>= 1) {
        if (threadIdx.x < w) part[threadIdx.x] += part[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) dg[h] = part[0];
}

// the forward state scan of the vector decay kind
template <int MODE, bool SAVE = false>
__global__ __launch_bounds__(kThreads) void mk_state_vec(Dims d, StateArgs sa) {
    extern __shared__ __align__(16) unsigned char smem[];
    state_scan_body<MODE, true, false, true, SAVE>(d, sa, blockIdx.x, gridDim.x, smem);
}

// the reverse scan alone (the states come from the forward call)
__global__ __launch_bounds__(kThreads) void mk_state_vec_rev(Dims d, StateArgs sa) {
    extern __shared__ __align__(16) unsigned char smem[];
    state_scan_body<2, true, true, true>(d, sa, blockIdx.x, gridDim.x, smem);
}

// both scans of the backward pass, vector decay kind (REM: also the remainder plane of S)
template <bool REM>
__global__ __launch_bounds__(kThreads) void mk_state_pair_vec(Dims d, StateArgs s1, StateArgs s2) {
    extern __shared__ __align__(16) unsigned char smem[];
    if (blockIdx.y == 0) state_scan_body<1, true, REM, true>(d, s1, blockIdx.x, gridDim.x, smem);
    else state_scan_body<2, true, REM, true>(d, s2, blockIdx.x, gridDim.x, smem);
}

#include "lsm_mfma_vec.h"
#include "lsm_mfma_walk.h"
#include "lsm_mfma_delta.h"

struct Ws {
    uint16_t *states, *dstates, *states_rem, *dstates_t, *dstates_rem;
    uint16_t* states_t;  // what the forward output kernel reads (S^T [v][i]); = states unless the states are saved
    float *dg_tok, *wdec, *winc, *lam;
    // vector decay: decayed operand planes [BH*T][128], chunk decay totals [BH*N][128], scores [BH*N][64][64]
    uint16_t *khat_hi, *khat_lo, *qhat_hi, *qhat_lo, *p_hi, *p_lo;
    float* lamv;
    size_t bytes;
};

// With saved states (d.save) the forward and the backward call share one workspace: the backward
// carving, followed by the plane of transposed states that only the forward call uses.
Ws carve(const Dims& d, void* ws, bool bwd) {
    char* p = static_cast<char*>(ws);
    size_t off = 0;
    Ws w{};
    // Planes are read and written at the same relative offsets by the same workgroups.  Plane sizes are
    // powers of two for the usual shapes, and starts that far apart map equal offsets to the same memory
    // channels (measured: the scan that writes three planes ran a third slower at such a placement), so
    // every plane is followed by a pad that moves the next one to other channels.
    constexpr size_t kSkew = 17 * 256;
    const size_t st = align256(size_t(d.BH()) * (d.dv / D) * d.N * D * D * 2) + kSkew;
    if (d.save) bwd = true;
    w.states = reinterpret_cast<uint16_t*>(p + off); off += st;
    w.states_t = w.states;
    if (d.kind == 3) {
        if (bwd) {
            w.dstates = reinterpret_cast<uint16_t*>(p + off); off += st;
            w.dstates_t = reinterpret_cast<uint16_t*>(p + off); off += st;
            w.states_rem = reinterpret_cast<uint16_t*>(p + off); off += align256(st / 2) + kSkew;  // one byte per element
            w.dstates_rem = reinterpret_cast<uint16_t*>(p + off); off += align256(st / 2) + kSkew;
        }
        const size_t plane = align256(size_t(d.BH()) * d.T * D * 2) + kSkew, sc = align256(size_t(d.BH()) * d.N * C * C * 2) + kSkew;
        uint16_t** planes[4] = {&w.khat_hi, &w.khat_lo, &w.qhat_hi, &w.qhat_lo};
        for (auto pp : planes) { *pp = reinterpret_cast<uint16_t*>(p + off); off += plane; }
        w.p_hi = reinterpret_cast<uint16_t*>(p + off); off += sc;
        w.p_lo = reinterpret_cast<uint16_t*>(p + off); off += sc;
        w.lamv = reinterpret_cast<float*>(p + off); off += align256(size_t(d.BH()) * d.N * D * 4);
        if (d.save) { w.states_t = reinterpret_cast<uint16_t*>(p + off); off += st; }
        w.bytes = off;
        return w;
    }
    if (bwd) { w.dstates = reinterpret_cast<uint16_t*>(p + off); off += st; }
    if (bwd && d.kind != 0) { w.states_rem = reinterpret_cast<uint16_t*>(p + off); off += align256(st / 2) + kSkew; }  // one byte per element
    if (d.kind != 0) {
        w.wdec = reinterpret_cast<float*>(p + off); off += align256(size_t(d.BH()) * d.N * C * 4);
        w.winc = reinterpret_cast<float*>(p + off); off += align256(size_t(d.BH()) * d.N * C * 4);
        w.lam = reinterpret_cast<float*>(p + off); off += align256(size_t(d.BH()) * d.N * 4);
    }
    if (bwd && d.kind == 1) { w.dg_tok = reinterpret_cast<float*>(p + off); off += align256(size_t(d.BH()) * d.N * 4); }  // per-chunk sums
    if (d.save) { w.states_t = reinterpret_cast<uint16_t*>(p + off); off += st; }
    w.bytes = off;
    return w;
}


// ---- fused walkers (scalar decay kinds): segment plan and workspace
// Segments per sequence: enough workgroups to give every compute unit two (the walkers fit two to a
// unit, and one hides the other's waits), no more (each extra segment adds a share of the summary pass).  m = chunks per segment.
constexpr int kWalkTargetWgs = 512;
struct SegPlan { int m, nseg; };
SegPlan seg_plan(const Dims& d) {
    const int nmax = (d.T + C - 1) / C;  // chunks of the longest possible sequence
    int nseg = (kWalkTargetWgs + d.seqs() - 1) / d.seqs();
    nseg = nseg < 1 ? 1 : (nseg > nmax ? nmax : nseg);
    const int m = (nmax + nseg - 1) / nseg;
    return SegPlan{m, (nmax + m - 1) / m};
}
// The reverse scan of the state gradients has four workgroups per sequence.  With fewer than one per compute
// unit it is cut into segments as well: `per` of the walkers' segments to each of its own, entry gradients from a
// summary pass of the reverse direction.
struct RevPlan { int per, nseg; };
RevPlan rev_plan(const Dims& d, const SegPlan& sp) {
    const int wgs = D / 32 * d.seqs();
    if (wgs >= 256 || sp.nseg <= 1) return RevPlan{sp.nseg, 1};
    const int want = (256 + wgs - 1) / wgs;  // one workgroup per compute unit: with two, the four strips of a sequence fall out of step and stop sharing their rows in L2
    const int per = sp.nseg / want > 1 ? sp.nseg / want : 1;
    return RevPlan{per, (sp.nseg + per - 1) / per};
}
struct WalkWs {
    float *bound_f, *gseg_f;     // entry states of the segments (forward in time) and the segments' total log-decays
    float *bound_r, *gseg_r;     // backward, segmented reverse scan only: the same for the state gradients, backward in time
    uint16_t* dstates;           // backward: one state gradient per chunk (fragment-major bf16)
    float *wdec, *winc, *lam;    // backward: decay tables of the reverse scan
    float* dgc;                  // per-head kind: per-chunk sums of dg
    size_t bytes;
    uint16_t* part[4];  // d_v = 256: the first value-slice pass's dq and dk (head, remainder), [BH*T][128] each
};
// The forward part comes first, at the same offsets in both carvings: with saved states the backward
// call finds the entry states where the forward call left them.
WalkWs carve_walk(const Dims& d, void* ws, bool bwd) {
    char* p = static_cast<char*>(ws);
    size_t off = 0;
    WalkWs w{};
    const SegPlan sp = seg_plan(d);
    auto take = [&](size_t bytes) { float* r = reinterpret_cast<float*>(p + off); off += align256(bytes); return r; };
    const size_t nb = sp.nseg > 1 ? size_t(d.seqs()) * sp.nseg * D * D * 4 : 0, ng = sp.nseg > 1 ? size_t(d.seqs()) * sp.nseg * 4 : 0;
    w.bound_f = take(nb);
    w.gseg_f = take(ng);
    if (bwd) {
        w.dstates = reinterpret_cast<uint16_t*>(take(size_t(d.BH()) * d.N * D * D * 2));
        if (d.kind != 0) {
            w.wdec = take(size_t(d.BH()) * d.N * C * 4);
            w.winc = take(size_t(d.BH()) * d.N * C * 4);
            w.lam = take(size_t(d.BH()) * d.N * 4);
        }
        if (d.kind == 1) w.dgc = take(size_t(d.BH()) * d.N * 4);
        if (rev_plan(d, sp).nseg > 1) {
            w.bound_r = take(nb);
            w.gseg_r = take(ng);
        }
        if (d.dv > D) {  // two value-slice passes: the first pass's dq and dk, head and remainder
            for (auto& pl : w.part) pl = reinterpret_cast<uint16_t*>(take(size_t(d.BH()) * d.T * D * 2));
        }
    }
    w.bytes = off;
    return w;
}

// Raise a kernel's dynamic LDS limit, once per kernel and device (every kernel is always launched with the
// same size, so the first call settles it).  The record is keyed by the kernel's address: instantiations of one
// kernel template share a function type, so a flag per type would let the first of them speak for all.
template <typename K>
hipError_t allow_lds(K kernel, int bytes) {
    struct Seen { const void* fn; uint64_t devices; };
    static std::mutex mu;
    static std::vector<Seen> seen;
    const void* fn = reinterpret_cast<const void*>(kernel);
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const uint64_t bit = uint64_t(1) << (dev & 63);
    {
        std::lock_guard<std::mutex> lk(mu);
        for (const Seen& x : seen)
            if (x.fn == fn && (x.devices & bit)) return hipSuccess;
    }
    e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> lk(mu);
    for (Seen& x : seen)
        if (x.fn == fn) { x.devices |= bit; return hipSuccess; }
    seen.push_back(Seen{fn, bit});
    return hipSuccess;
}

}  // namespace

bool mfma_supported(const Dims& d) {
    // d_v: any multiple of 128.  The vector kind scans each 128-wide value slice as a sequence of its own; the scalar
    // kinds run their walkers once per slice (the value columns of the state evolve independently).
    return d.bf16 && d.C == C && d.dk == D && d.dv % D == 0 && (d.kind == 3 || d.dv <= 2 * D);
}
bool mfma_bwd_supported(const Dims& d) { return mfma_supported(d); }

size_t mfma_fwd_workspace(const Dims& d) { return d.kind == 3 ? carve(d, nullptr, false).bytes : carve_walk(d, nullptr, d.save).bytes; }
// chunk states and decay tables of the intra-chunk benchmark aid
size_t mfma_intra_bench_workspace(const Dims& d0) {
    Dims d = d0;
    d.save = false;
    return carve(d, nullptr, false).bytes;
}
size_t mfma_bwd_workspace(const Dims& d) { return d.kind == 3 ? carve(d, nullptr, true).bytes : carve_walk(d, nullptr, true).bytes; }

namespace {
template <int MODE>
hipError_t launch_state(const Dims& d, hipStream_t st, const StateArgs& sa) {
    const dim3 sgrid(D / 32 * d.seqs() * (sa.seg_n > 1 ? sa.seg_n : 1)), block(kThreads);
    const int lds = kStateLdsNone;
    hipError_t e;
    if (d.kind == 0) {
        if ((e = allow_lds(mk_state_seq<MODE, false>, lds)) != hipSuccess) return e;
        hipLaunchKernelGGL((mk_state_seq<MODE, false>), sgrid, block, lds, st, d, sa);
    } else {
        if ((e = allow_lds(mk_state_seq<MODE, true>, lds)) != hipSuccess) return e;
        hipLaunchKernelGGL((mk_state_seq<MODE, true>), sgrid, block, lds, st, d, sa);
    }
    return hipSuccess;
}
void launch_prep(const Dims& d, hipStream_t st, const float* g, const Ws& w) {
    if (d.kind == 0) return;
    ProfScope ps(KID_MFMA_PREP, st);
    hipLaunchKernelGGL(mk_decay_prep, dim3(d.N, d.BH()), dim3(64), 0, st, d, g, w.wdec, w.winc, w.lam);
}
}  // namespace

namespace {
hipError_t launch_vec_prep(const Dims& d, hipStream_t st, const uint16_t* q, const uint16_t* k, const float* g, const Ws& w) {
    const hipError_t e = allow_lds(mk_vec_prep, kPrepLds);
    if (e != hipSuccess) return e;
    ProfScope ps(KID_MFMA_VEC_PREP, st);
    hipLaunchKernelGGL(mk_vec_prep, dim3(d.N, d.BH()), dim3(kThreads), kPrepLds, st, d, q, k, g, w.khat_hi, w.khat_lo,
                       w.qhat_hi, w.qhat_lo, w.lamv, w.p_hi, w.p_lo);
    return hipSuccess;
}

hipError_t vec_fwd(const Dims& d, const FwdArgs& a) {
    Ws w = carve(d, a.ws, false);
    auto q = static_cast<const uint16_t*>(a.q), k = static_cast<const uint16_t*>(a.k), v = static_cast<const uint16_t*>(a.v);
    const int nvh = d.dv / D;
    hipError_t e;
    if ((e = launch_vec_prep(d, a.stream, q, k, a.g, w)) != hipSuccess) return e;
    {
        ProfScope ps(KID_MFMA_STATE, a.stream);
        if ((e = allow_lds(mk_state_vec<3>, kStateLdsPlain)) != hipSuccess) return e;
        const dim3 sgrid(D / 32 * d.seqs() * nvh);
        if (d.save) {
            if ((e = allow_lds(mk_state_vec<3, true>, kStateLdsPlain)) != hipSuccess) return e;
            StateArgs sa{v, w.khat_hi, nullptr, w.lamv, w.states_t, w.states_rem, a.m0, a.mT, w.khat_lo, d.dv, nvh, w.states};
            hipLaunchKernelGGL((mk_state_vec<3, true>), sgrid, dim3(kThreads), kStateLdsPlain, a.stream, d, sa);
        } else {
            StateArgs sa{v, w.khat_hi, nullptr, w.lamv, w.states, nullptr, a.m0, a.mT, w.khat_lo, d.dv, nvh};
            hipLaunchKernelGGL(mk_state_vec<3>, sgrid, dim3(kThreads), kStateLdsPlain, a.stream, d, sa);
        }
    }
    {
        ProfScope ps(KID_MFMA_OUTPUT, a.stream);
        if ((e = allow_lds(mk_output_vec<false>, kOutVecLds)) != hipSuccess) return e;
        hipLaunchKernelGGL(mk_output_vec<false>, dim3(d.N, d.BH(), nvh), dim3(kThreads), kOutVecLds, a.stream, d, w.qhat_hi, w.qhat_lo, v,
                           w.p_hi, w.p_lo, w.states_t, static_cast<uint16_t*>(a.o));
    }
    return hipGetLastError();
}
}  // namespace

namespace {
// ---- fused walkers: host side
// entry states of the segments of one direction: summary pass, then the scan over segments
template <bool REV>
hipError_t walk_bounds(const Dims& d, hipStream_t st, const SegPlan& sp, const uint16_t* xk, const uint16_t* xv, const float* g,
                       const float* edge_in, float* bound, float* gseg, int skip = 1, const uint16_t* xv_lo = nullptr) {
    if (sp.nseg <= 1) return hipSuccess;
    WalkArgs a{};
    a.xk = xk; a.xv = xv; a.g = g; a.bound = bound; a.gseg = gseg; a.m = sp.m; a.nseg = sp.nseg; a.skip = skip; a.xv_lo = xv_lo;
    hipError_t e;
    const dim3 grid(sp.nseg, d.seqs()), block(kThreads);
    {
        ProfScope ps(KID_WALK_SUMMARY, st);
        constexpr int lds = walk_lds(true);
        if (xv_lo) {  // values in two planes (delta-rule backward; forward direction only)
            constexpr int lds2 = lds + C * LD * 2;
            if (d.kind == 0) {
                if ((e = allow_lds(mk_walk<REV, false, true, true>, lds2)) != hipSuccess) return e;
                hipLaunchKernelGGL((mk_walk<REV, false, true, true>), grid, block, lds2, st, d, a);
            } else {
                if ((e = allow_lds(mk_walk<REV, true, true, true>, lds2)) != hipSuccess) return e;
                hipLaunchKernelGGL((mk_walk<REV, true, true, true>), grid, block, lds2, st, d, a);
            }
        } else if (d.kind == 0) {
            if ((e = allow_lds(mk_walk<REV, false, true>, lds)) != hipSuccess) return e;
            hipLaunchKernelGGL((mk_walk<REV, false, true>), grid, block, lds, st, d, a);
        } else {
            if ((e = allow_lds(mk_walk<REV, true, true>, lds)) != hipSuccess) return e;
            hipLaunchKernelGGL((mk_walk<REV, true, true>), grid, block, lds, st, d, a);
        }
    }
    ProfScope ps(KID_WALK_SCAN, st);
    hipLaunchKernelGGL(mk_bound_scan<REV>, dim3(D * D / kThreads, d.seqs()), block, 0, st, d, edge_in, bound, gseg, sp.m, sp.nseg, skip);
    return hipSuccess;
}

// One 128-wide slice of the value dimension (d.vm slices, this one d.vs; a single pass when d_v = 128).
hipError_t walk_fwd_slice(const Dims& d, const FwdArgs& a) {
    const WalkWs w = carve_walk(d, a.ws, false);
    const SegPlan sp = seg_plan(d);
    auto q = static_cast<const uint16_t*>(a.q), k = static_cast<const uint16_t*>(a.k), v = static_cast<const uint16_t*>(a.v);
    hipError_t e;
    if ((e = walk_bounds<false>(d, a.stream, sp, k, v, a.g, a.m0, w.bound_f, w.gseg_f)) != hipSuccess) return e;
    WalkArgs wa{};
    wa.xq = q; wa.xk = k; wa.xv = v; wa.g = a.g; wa.out = static_cast<uint16_t*>(a.o);
    wa.edge_in = a.m0; wa.edge_out = a.mT; wa.bound = w.bound_f; wa.m = sp.m; wa.nseg = sp.nseg;
    const dim3 grid(sp.nseg, d.seqs()), block(kThreads);
    constexpr int lds = walk_lds(false);
    ProfScope ps(KID_WALK_FWD, a.stream);
    if (d.kind == 0) {
        if ((e = allow_lds(mk_walk<false, false, false>, lds)) != hipSuccess) return e;
        hipLaunchKernelGGL((mk_walk<false, false, false>), grid, block, lds, a.stream, d, wa);
    } else {
        if ((e = allow_lds(mk_walk<false, true, false>, lds)) != hipSuccess) return e;
        hipLaunchKernelGGL((mk_walk<false, true, false>), grid, block, lds, a.stream, d, wa);
    }
    return hipGetLastError();
}
hipError_t walk_fwd(const Dims& d0, const FwdArgs& a) {
    Dims d = d0;
    d.vm = d0.dv / D;
    for (d.vs = 0; d.vs < d.vm; ++d.vs) {  // the passes share the workspace: same stream, one after the other
        const hipError_t e = walk_fwd_slice(d, a);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_walk_grad(const Dims& d, const SegPlan& sp, const GradArgs& ga, hipStream_t st) {
    const dim3 grid(sp.nseg, d.seqs()), block(kGrad8Threads);
    hipError_t e;
    ProfScope ps(KID_WALK_GRAD, st);
    if (ga.v_lo) {  // values in two planes (delta-rule backward)
        constexpr int lds = walk_grad_lds(true);
        if (d.kind == 0) {
            if ((e = allow_lds(mk_walk_grad<false, false, true>, lds)) != hipSuccess) return e;
            hipLaunchKernelGGL((mk_walk_grad<false, false, true>), grid, block, lds, st, d, ga);
        } else {
            if ((e = allow_lds(mk_walk_grad<true, true, true>, lds)) != hipSuccess) return e;
            hipLaunchKernelGGL((mk_walk_grad<true, true, true>), grid, block, lds, st, d, ga);
        }
        return hipSuccess;
    }
    // d_v = 256: pass 0 leaves dq and dk in the partial planes (WIDE 1), pass 1 adds them to its own (WIDE 2)
    const int wide = d.vm == 1 ? 0 : (d.vs == 0 ? 1 : 2);
    auto launch = [&](auto kernel) -> hipError_t {
        const hipError_t le = allow_lds(kernel, kWalkGradLds);
        if (le != hipSuccess) return le;
        hipLaunchKernelGGL(kernel, grid, block, kWalkGradLds, st, d, ga);
        return hipSuccess;
    };
    auto pick = [&](auto w0, auto w1, auto w2) { return wide == 0 ? launch(w0) : wide == 1 ? launch(w1) : launch(w2); };
    if (d.kind == 0)
        return pick(mk_walk_grad<false, false, false, 0>, mk_walk_grad<false, false, false, 1>, mk_walk_grad<false, false, false, 2>);
    if (!ga.dg_tok)
        return pick(mk_walk_grad<true, false, false, 0>, mk_walk_grad<true, false, false, 1>, mk_walk_grad<true, false, false, 2>);
    return pick(mk_walk_grad<true, true, false, 0>, mk_walk_grad<true, true, false, 1>, mk_walk_grad<true, true, false, 2>);
}

hipError_t walk_bwd_slice(const Dims& d, const BwdArgs& a) {
    const WalkWs w = carve_walk(d, a.ws, true);
    const SegPlan sp = seg_plan(d);
    auto q = static_cast<const uint16_t*>(a.q), k = static_cast<const uint16_t*>(a.k), v = static_cast<const uint16_t*>(a.v);
    auto d_o = static_cast<const uint16_t*>(a.d_o);
    hipError_t e;
    // state gradients: the reverse scan leaves one per chunk (and d_init_state)
    if (d.kind != 0 && d.vs == 0) {  // the decay tables are the same for every value slice
        ProfScope ps(KID_MFMA_PREP, a.stream);
        hipLaunchKernelGGL(mk_decay_prep, dim3(d.N, d.BH()), dim3(64), 0, a.stream, d, a.g, w.wdec, w.winc, w.lam);
    }
    {
        StateArgs sa{d_o, q, w.winc, w.lam, w.dstates, nullptr, a.d_mT, a.d_m0};
        const RevPlan rp = rev_plan(d, sp);
        if (rp.nseg > 1) {
            // entry gradients of the segments: the summary pass and the segment scan, backward in time (roles: key = q,
            // value = d_o)
            if ((e = walk_bounds<true>(d, a.stream, sp, q, d_o, a.g, a.d_mT, w.bound_r, w.gseg_r, rp.per)) != hipSuccess) return e;
            sa.seg_bound = w.bound_r;
            sa.seg_m = rp.per * sp.m; sa.seg_n = rp.nseg; sa.fine_m = sp.m; sa.fine_n = sp.nseg;
        }
        ProfScope ps(KID_MFMA_DSTATE, a.stream);
        if ((e = launch_state<2>(d, a.stream, sa)) != hipSuccess) return e;
    }
    // entry states of the segments, unless the forward call left them
    if (!d.save && (e = walk_bounds<false>(d, a.stream, sp, k, v, a.g, a.m0, w.bound_f, w.gseg_f)) != hipSuccess) return e;
    GradArgs ga{q, k, v, d_o, a.g, w.dstates, static_cast<uint16_t*>(a.dq), static_cast<uint16_t*>(a.dk), static_cast<uint16_t*>(a.dv),
                a.dg ? (d.kind == 1 ? w.dgc : a.dg) : nullptr, a.m0, w.bound_f, sp.m, sp.nseg};
    for (int i = 0; i < 4; ++i) ga.part[i] = w.part[i];
    const dim3 block(kThreads);
    // the gradient walker holds one workgroup per compute unit, the forward walker two: where the plan gives every unit
    // two workgroups, the gradient walker takes segments of twice the length (half as many state loads and prologues)
    SegPlan gp = sp;
    if (sp.nseg % 2 == 0 && sp.nseg * d.seqs() >= 512) {
        gp = SegPlan{sp.m * 2, sp.nseg / 2};
        ga.m = gp.m; ga.nseg = gp.nseg; ga.bound_per = 2; ga.bound_n = sp.nseg;
    }
    if ((e = launch_walk_grad(d, gp, ga, a.stream)) != hipSuccess) return e;
    if (a.dg && d.kind == 1 && d.vs == d.vm - 1) {  // after the last slice has added its share
        ProfScope ps(KID_HEAD_REDUCE, a.stream);
        hipLaunchKernelGGL(mk_head_reduce, dim3(d.H), block, 0, a.stream, d, w.dgc, a.dg);
    }
    return hipGetLastError();
}
hipError_t walk_bwd(const Dims& d0, const BwdArgs& a) {
    Dims d = d0;
    d.vm = d0.dv / D;
    for (d.vs = 0; d.vs < d.vm; ++d.vs) {  // dq, dk and the decay gradient sum over the slices: later passes add to them
        const hipError_t e = walk_bwd_slice(d, a);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}
}  // namespace

hipError_t mfma_fwd(const Dims& d, const FwdArgs& a) {
    if (d.kind == 3) return vec_fwd(d, a);
    return walk_fwd(d, a);
}

namespace {
hipError_t vec_bwd(const Dims& d, const BwdArgs& a) {
    hipError_t e;
    Ws w = carve(d, a.ws, true);
    auto q = static_cast<const uint16_t*>(a.q), k = static_cast<const uint16_t*>(a.k), v = static_cast<const uint16_t*>(a.v);
    auto d_o = static_cast<const uint16_t*>(a.d_o);
    const int nvh = d.dv / D;
    if (!d.save && (e = launch_vec_prep(d, a.stream, q, k, a.g, w)) != hipSuccess) return e;
    if (d.save) {  // the decayed operand planes, the scores and the states are the forward call's
        ProfScope ps(KID_MFMA_DSTATE, a.stream);
        const StateArgs s2{d_o, w.qhat_hi, nullptr, w.lamv, w.dstates, a.dg ? w.dstates_rem : nullptr, a.d_mT, a.d_m0,
                           w.qhat_lo, d.dv, nvh, w.dstates_t};
        if ((e = allow_lds(mk_state_vec_rev, kStateLdsPlain)) != hipSuccess) return e;
        hipLaunchKernelGGL(mk_state_vec_rev, dim3(D / 32 * d.seqs() * nvh), dim3(kThreads), kStateLdsPlain, a.stream, d, s2);
    } else {
        ProfScope ps(KID_MFMA_STATE_BWD, a.stream);
        const StateArgs s1{v, w.khat_hi, nullptr, w.lamv, w.states, a.dg ? w.states_rem : nullptr, a.m0, nullptr,
                           w.khat_lo, d.dv, nvh};
        const StateArgs s2{d_o, w.qhat_hi, nullptr, w.lamv, w.dstates, a.dg ? w.dstates_rem : nullptr, a.d_mT, a.d_m0,
                           w.qhat_lo, d.dv, nvh, w.dstates_t};
        const dim3 sgrid(D / 32 * d.seqs() * nvh, 2);
        if (a.dg) {
            if ((e = allow_lds(mk_state_pair_vec<true>, kStateLdsPlain)) != hipSuccess) return e;
            hipLaunchKernelGGL(mk_state_pair_vec<true>, sgrid, dim3(kThreads), kStateLdsPlain, a.stream, d, s1, s2);
        } else {
            if ((e = allow_lds(mk_state_pair_vec<false>, kStateLdsPlain)) != hipSuccess) return e;
            hipLaunchKernelGGL(mk_state_pair_vec<false>, sgrid, dim3(kThreads), kStateLdsPlain, a.stream, d, s1, s2);
        }
    }
    {
        ProfScope ps(KID_MFMA_VEC_DV, a.stream);
        if ((e = allow_lds(mk_output_vec<true>, kOutVecLds)) != hipSuccess) return e;
        hipLaunchKernelGGL(mk_output_vec<true>, dim3(d.N, d.BH(), nvh), dim3(kThreads), kOutVecLds, a.stream, d, w.khat_hi,
                           w.khat_lo, d_o, w.p_hi, w.p_lo, w.dstates_t, static_cast<uint16_t*>(a.dv));
    }
    {
        ProfScope ps(KID_MFMA_GRAD, a.stream);
        if ((e = allow_lds(mk_grad_vec, kGradVecLds)) != hipSuccess) return e;
        hipLaunchKernelGGL(mk_grad_vec, dim3(d.N, d.BH()), dim3(kGradVecThreads), kGradVecLds, a.stream, d, q, k, v, d_o, a.g,
                           w.states, a.dg ? w.states_rem : nullptr, w.dstates, w.dstates_rem, static_cast<uint16_t*>(a.dq),
                           static_cast<uint16_t*>(a.dk), a.dg);
    }
    return hipGetLastError();
}
}  // namespace

hipError_t mfma_intra_bench(const Dims& d0, const FwdArgs& a, int reps) {
    if (d0.kind == 3 || d0.dv != D || !mfma_supported(d0)) return hipErrorInvalidValue;
    Dims d = d0;
    d.save = false;
    Ws w = carve(d, a.ws, false);
    hipError_t e;
    if ((e = allow_lds(mk_output<true>, kOutLdsRepeat)) != hipSuccess) return e;
    // the per-chunk kernel reads materialised chunk states: decay tables and the chunk-state scan first
    launch_prep(d, a.stream, a.g, w);
    const StateArgs sa{static_cast<const uint16_t*>(a.k), static_cast<const uint16_t*>(a.v), w.wdec, w.lam, w.states, nullptr, a.m0, nullptr};
    if ((e = launch_state<0>(d, a.stream, sa)) != hipSuccess) return e;
    ProfScope ps(KID_MFMA_OUTPUT, a.stream);
    hipLaunchKernelGGL(mk_output<true>, dim3(d.N, d.BH()), dim3(kThreads), kOutLdsRepeat, a.stream, d,
                       static_cast<const uint16_t*>(a.q), static_cast<const uint16_t*>(a.k),
                       static_cast<const uint16_t*>(a.v), a.g, w.states, static_cast<uint16_t*>(a.o), reps);
    return hipGetLastError();
}

// ---- delta-rule rows: host side
bool delta_supported(const Dims& d) { return d.bf16 && d.C == C && d.dk == D && d.dv == D && (d.kind == 0 || d.kind == 2); }
namespace {
struct DeltaWs;
DeltaWs carve_delta(const Dims& d, void* ws);
size_t carve_delta_bytes(const Dims& d);
// Segments of the delta walkers: one workgroup per compute unit is the most they can use, so a sequence is cut only
// when there are clearly fewer sequences than units.
SegPlan delta_plan(const Dims& d) {
    const int nmax = (d.T + C - 1) / C;
    int nseg = d.seqs() >= 192 ? 1 : (256 + d.seqs() - 1) / d.seqs();
    nseg = nseg > nmax ? nmax : nseg;
    const int m = (nmax + nseg - 1) / nseg;
    return SegPlan{m, (nmax + m - 1) / m};
}
// sum A | sum B | entry states, [seqs][nseg][128 x 128] fp32 each (nothing for a single segment)
size_t delta_seg_bytes(const Dims& d) {
    const SegPlan sp = delta_plan(d);
    return sp.nseg > 1 ? 3 * align256(size_t(d.seqs()) * sp.nseg * D * D * 4) : 0;
}
}  // namespace
// Dims::save: the forward call also leaves T^T and the pseudo-values in the workspace, laid out as the backward call
// carves it, and the backward call does not run the prep and the walk again.
size_t delta_fwd_workspace(const Dims& d) {
    if (d.save) return carve_delta_bytes(d);
    return align256(size_t(d.BH()) * d.T * D * 2) + align256(size_t(d.BH()) * d.T * D * 4) + delta_seg_bytes(d);
}
namespace {
hipError_t launch_delta_fwd(const Dims& d, const DeltaPrepArgs& pa, DeltaWalkArgs wa, void* segws, hipStream_t stream);
}
hipError_t delta_fwd_saving(const Dims& d, const DeltaArgs& a);
hipError_t delta_fwd(const Dims& d, const DeltaArgs& a) {
    if (d.save) return delta_fwd_saving(d, a);
    char* p = static_cast<char*>(a.ws);
    uint16_t* what = reinterpret_cast<uint16_t*>(p);
    float* uhat = reinterpret_cast<float*>(p + align256(size_t(d.BH()) * d.T * D * 2));
    auto q = static_cast<const uint16_t*>(a.q), k = static_cast<const uint16_t*>(a.k), v = static_cast<const uint16_t*>(a.v);
    const DeltaPrepArgs pa{k, v, a.log_alpha, a.beta, a.bw, what, uhat, nullptr};
    const DeltaWalkArgs wa{q, k, what, uhat, a.log_alpha, static_cast<uint16_t*>(a.o), a.m0, a.mT, nullptr, nullptr};
    return launch_delta_fwd(d, pa, wa, p + align256(size_t(d.BH()) * d.T * D * 2) + align256(size_t(d.BH()) * d.T * D * 4), a.stream);
}
namespace {
template <bool DEC>
hipError_t launch_delta_fwd_t(const Dims& d, const DeltaPrepArgs& pa, DeltaWalkArgs wa, void* segws, hipStream_t st) {
    hipError_t e;
    const SegPlan sp = delta_plan(d);
    const dim3 pgrid(d.N, d.BH()), wgrid(sp.nseg, d.seqs()), block(kThreads);
    if ((e = allow_lds(mk_delta_prep<DEC>, kDeltaPrepLds)) != hipSuccess) return e;
    if ((e = allow_lds(mk_delta_walk8<DEC, 0>, kDeltaWalk8Lds)) != hipSuccess) return e;
    {
        ProfScope ps(KID_DELTA_PREP, st);
        hipLaunchKernelGGL(mk_delta_prep<DEC>, pgrid, block, kDeltaPrepLds, st, d, pa);
    }
    wa.m = sp.m;
    wa.nseg = sp.nseg;
    if (sp.nseg > 1) {
        const size_t one = align256(size_t(d.seqs()) * sp.nseg * D * D * 4);
        float* sumA = reinterpret_cast<float*>(segws);
        float* sumB = reinterpret_cast<float*>(static_cast<char*>(segws) + one);
        float* bound = reinterpret_cast<float*>(static_cast<char*>(segws) + 2 * one);
        if ((e = allow_lds(mk_delta_walk8<DEC, 1>, kDeltaWalk8Lds)) != hipSuccess) return e;
        if ((e = allow_lds(mk_delta_walk8<DEC, 2>, kDeltaWalk8Lds)) != hipSuccess) return e;
        if ((e = allow_lds(mk_delta_combine<false>, kDeltaCombineLds)) != hipSuccess) return e;
        {
            ProfScope ps(KID_DELTA_SUMMARY, st);
            DeltaWalkArgs sa = wa;
            sa.sum = sumB;
            hipLaunchKernelGGL((mk_delta_walk8<DEC, 1>), wgrid, dim3(512), kDeltaWalk8Lds, st, d, sa);
        }
        {
            ProfScope ps(KID_DELTA_SUMMARY, st);
            DeltaWalkArgs sa = wa;
            sa.sum = sumA;
            hipLaunchKernelGGL((mk_delta_walk8<DEC, 2>), wgrid, dim3(512), kDeltaWalk8Lds, st, d, sa);
        }
        {
            ProfScope ps(KID_DELTA_COMBINE, st);
            hipLaunchKernelGGL(mk_delta_combine<false>, dim3(d.seqs()), block, kDeltaCombineLds, st, d, wa.edge_in, sumA, sumB, bound, sp.m, sp.nseg);
        }
        wa.bound = bound;
    }
    ProfScope ps(KID_DELTA_WALK, st);
    hipLaunchKernelGGL((mk_delta_walk8<DEC, 0>), wgrid, dim3(512), kDeltaWalk8Lds, st, d, wa);
    return hipGetLastError();
}
hipError_t launch_delta_fwd(const Dims& d, const DeltaPrepArgs& pa, DeltaWalkArgs wa, void* segws, hipStream_t stream) {
    return d.kind == 0 ? launch_delta_fwd_t<false>(d, pa, wa, segws, stream) : launch_delta_fwd_t<true>(d, pa, wa, segws, stream);
}

template <bool DEC>
hipError_t launch_delta_rwalk(const Dims& d, DeltaRevArgs ra, void* segws, hipStream_t st) {
    hipError_t e;
    const SegPlan sp = delta_plan(d);
    const dim3 grid(sp.nseg, d.seqs()), block(kThreads);
    if ((e = allow_lds(mk_delta_rwalk<DEC, 0>, kDeltaRevLds)) != hipSuccess) return e;
    ra.m = sp.m;
    ra.nseg = sp.nseg;
    if (sp.nseg > 1) {
        const size_t one = align256(size_t(d.seqs()) * sp.nseg * D * D * 4);
        float* sumA = reinterpret_cast<float*>(segws);
        float* sumB = reinterpret_cast<float*>(static_cast<char*>(segws) + one);
        float* bound = reinterpret_cast<float*>(static_cast<char*>(segws) + 2 * one);
        if ((e = allow_lds(mk_delta_rwalk<DEC, 1>, kDeltaRevLds)) != hipSuccess) return e;
        if ((e = allow_lds(mk_delta_rwalk<DEC, 2>, kDeltaRevLds)) != hipSuccess) return e;
        if ((e = allow_lds(mk_delta_combine<true>, kDeltaCombineLds)) != hipSuccess) return e;
        {
            ProfScope ps(KID_DELTA_SUMMARY, st);
            DeltaRevArgs sa = ra;
            sa.sum = sumB;
            hipLaunchKernelGGL((mk_delta_rwalk<DEC, 1>), grid, block, kDeltaRevLds, st, d, sa);
        }
        {
            ProfScope ps(KID_DELTA_SUMMARY, st);
            DeltaRevArgs sa = ra;
            sa.sum = sumA;
            hipLaunchKernelGGL((mk_delta_rwalk<DEC, 2>), grid, block, kDeltaRevLds, st, d, sa);
        }
        {
            ProfScope ps(KID_DELTA_COMBINE, st);
            hipLaunchKernelGGL(mk_delta_combine<true>, dim3(d.seqs()), block, kDeltaCombineLds, st, d, ra.edge_in, sumA, sumB, bound, sp.m, sp.nseg);
        }
        ra.bound = bound;
    }
    ProfScope ps(KID_DELTA_RWALK, st);
    hipLaunchKernelGGL((mk_delta_rwalk<DEC, 0>), grid, block, kDeltaRevLds, st, d, ra);
    return hipSuccess;
}

struct DeltaWs {
    uint16_t *what, *tt, *usave, *usave_l, *dstates, *du_h, *du_l, *dw_h, *dw_l;
    float* uhat;
    void* walk;   // bound_f, gseg_f of the gradient walker
    void* seg;    // segment summaries and entry states of the delta walker
    void* seg_r;  // the same for the reverse walker
    size_t bytes;
};
DeltaWs carve_delta(const Dims& d, void* ws) {
    char* p = static_cast<char*>(ws);
    size_t off = 0;
    auto take = [&](size_t bytes) { char* r = p + off; off += align256(bytes); return r; };
    const size_t rows = size_t(d.BH()) * d.T;
    DeltaWs w{};
    w.what = reinterpret_cast<uint16_t*>(take(rows * D * 2));
    w.uhat = reinterpret_cast<float*>(take(rows * D * 4));
    w.tt = reinterpret_cast<uint16_t*>(take(size_t(d.BH()) * d.N * 2 * C * C * 2));
    w.usave = reinterpret_cast<uint16_t*>(take(rows * D * 2));
    w.usave_l = reinterpret_cast<uint16_t*>(take(rows * D * 2));
    w.dstates = reinterpret_cast<uint16_t*>(take(size_t(d.BH()) * d.N * D * D * 2));
    w.du_h = reinterpret_cast<uint16_t*>(take(rows * D * 2));
    w.du_l = reinterpret_cast<uint16_t*>(take(rows * D * 2));
    w.dw_h = reinterpret_cast<uint16_t*>(take(rows * D * 2));
    w.dw_l = reinterpret_cast<uint16_t*>(take(rows * D * 2));
    w.walk = p + off;
    off += carve_walk(d, nullptr, false).bytes;
    w.seg = p + off;
    off += delta_seg_bytes(d);
    w.seg_r = p + off;
    off += delta_seg_bytes(d);
    w.bytes = off;
    return w;
}
size_t carve_delta_bytes(const Dims& d) { return carve_delta(d, nullptr).bytes; }
}  // namespace
size_t delta_bwd_workspace(const Dims& d) { return carve_delta(d, nullptr).bytes; }

hipError_t delta_fwd_saving(const Dims& d, const DeltaArgs& a) {
    const DeltaWs w = carve_delta(d, a.ws);
    auto q = static_cast<const uint16_t*>(a.q), k = static_cast<const uint16_t*>(a.k), v = static_cast<const uint16_t*>(a.v);
    const DeltaPrepArgs pa{k, v, a.log_alpha, a.beta, a.bw, w.what, w.uhat, w.tt};
    const DeltaWalkArgs wa{q, k, w.what, w.uhat, a.log_alpha, static_cast<uint16_t*>(a.o), a.m0, a.mT, w.usave, w.usave_l};
    return launch_delta_fwd(d, pa, wa, w.seg, a.stream);
}

hipError_t delta_bwd(const Dims& d, const DeltaBwdArgs& a) {
    const DeltaWs w = carve_delta(d, a.ws);
    const WalkWs ww = carve_walk(d, w.walk, false);
    const SegPlan sp = seg_plan(d);
    auto q = static_cast<const uint16_t*>(a.q), k = static_cast<const uint16_t*>(a.k), v = static_cast<const uint16_t*>(a.v);
    auto d_o = static_cast<const uint16_t*>(a.d_o);
    hipError_t e;
    // forward again: What, Uhat, T, and the pseudo-values U in the layout of v
    if (!d.save) {
        const DeltaPrepArgs pa{k, v, a.log_alpha, a.beta, a.bw, w.what, w.uhat, w.tt};
        const DeltaWalkArgs wa{q, k, w.what, w.uhat, a.log_alpha, nullptr, a.m0, nullptr, w.usave, w.usave_l};
        if ((e = launch_delta_fwd(d, pa, wa, w.seg, a.stream)) != hipSuccess) return e;
    }
    // state gradients and dU, backward in time
    {
        const DeltaRevArgs ra{q, k, d_o, w.what, a.log_alpha, w.dstates, w.du_h, w.du_l, a.d_mT, a.d_m0};
        e = d.kind == 0 ? launch_delta_rwalk<false>(d, ra, w.seg_r, a.stream) : launch_delta_rwalk<true>(d, ra, w.seg_r, a.stream);
        if (e != hipSuccess) return e;
    }
    // with U as the values the recurrence is the scalar-decay one: dq, the key gradient through scores and state update
    // and the decay gradient of those terms from the gradient walker (its value gradient is dU once more, not wanted)
    if ((e = walk_bounds<false>(d, a.stream, sp, k, w.usave, a.log_alpha, a.m0, ww.bound_f, ww.gseg_f, 1, w.usave_l)) != hipSuccess) return e;
    GradArgs ga{q, k, w.usave, d_o, a.log_alpha, w.dstates, static_cast<uint16_t*>(a.dq), static_cast<uint16_t*>(a.dk),
                static_cast<uint16_t*>(a.dv), d.kind == 0 ? nullptr : a.d_log_alpha, a.m0, ww.bound_f, sp.m, sp.nseg, w.usave_l, w.du_h, w.du_l, w.dw_h, w.dw_l};
    // dk <- head, dv <- remainder of its key gradient; it also leaves dW = -dU S^T, the gradient of What
    if ((e = launch_walk_grad(d, sp, ga, a.stream)) != hipSuccess) return e;
    // everything that goes through the triangular solve, chunk by chunk; completes dk, dv and the parameter gradients
    {
        const DeltaGradArgs g3{k, v, w.du_h, w.du_l, w.dw_h, w.dw_l, w.tt, a.log_alpha, a.beta, a.bw,
                               static_cast<const uint16_t*>(a.dk), static_cast<const uint16_t*>(a.dv),
                               static_cast<uint16_t*>(a.dk), static_cast<uint16_t*>(a.dv), a.d_log_alpha, a.d_beta, a.d_bw};
        const int jobs = d.N * d.BH();
        const dim3 grid(jobs < 256 ? jobs : 256);
        ProfScope ps(KID_DELTA_GRAD, a.stream);
        if (d.kind == 0) {
            if ((e = allow_lds(mk_delta_grad<false>, kDeltaGradLds)) != hipSuccess) return e;
            hipLaunchKernelGGL(mk_delta_grad<false>, grid, dim3(kThreads), kDeltaGradLds, a.stream, d, g3);
        } else {
            if ((e = allow_lds(mk_delta_grad<true>, kDeltaGradLds)) != hipSuccess) return e;
            hipLaunchKernelGGL(mk_delta_grad<true>, grid, dim3(kThreads), kDeltaGradLds, a.stream, d, g3);
        }
    }
    return hipGetLastError();
}

hipError_t mfma_bwd(const Dims& d, const BwdArgs& a) {
    if (d.kind == 3) return vec_bwd(d, a);
    return walk_bwd(d, a);
}

}  // namespace lsm
