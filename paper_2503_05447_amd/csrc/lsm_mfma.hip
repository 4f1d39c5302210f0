// MFMA kernel family of the chunkwise LSM path for gfx950: bf16 operands, fp32 accumulation,
// chunk = 64 tokens, d_k = d_v = 128, decay kinds none / per-head / per-token scalar.
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
// A contraction over tokens needs a token-major tile with tokens along k.  Tiles arrive
// feature-contiguous, so they are turned with an MFMA against the identity: D = X * I leaves
// lane (n, half) with 16 tokens of feature n, which (a) is written to LDS as 8-byte pieces of a
// transposed tile, or (b) is used directly as an operand, the partner operand then reading its k
// index in the same permuted order ("perm" fragments below).  Decay weights are applied to the
// fp32 values of that step, before the single rounding to bf16.
#include "lsm_internal.h"

namespace lsm {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int C = 64;      // tokens per chunk
constexpr int D = 128;     // d_k = d_v
constexpr int LD = D + 8;  // row stride (elements) of a [*, 128] bf16 tile in LDS: 68 words, == 4 mod 32
constexpr int LDP = C + 8; // row stride of a [*, 64] bf16 tile in LDS: 36 words, == 4 mod 32
constexpr int kThreads = 256;

__device__ __forceinline__ f32x16 mfma(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    f32x2 f = {lo, hi};
    bf16x2 h = __builtin_convertvector(f, bf16x2);
    return __builtin_bit_cast(uint32_t, h);
}
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// 8 consecutive bf16 of row `row` starting at column `col` (16-byte aligned)
__device__ __forceinline__ bf16x8 frag(const uint16_t* tile, int ld, int row, int col) {
    return *reinterpret_cast<const bf16x8*>(tile + row * ld + col);
}
// k index in the permuted order of a D-layout operand: columns col0 + 4*half + {0..3} and col0 + 8 + 4*half + {0..3}
__device__ __forceinline__ bf16x8 frag_perm(const uint16_t* tile, int ld, int row, int col0, int half) {
    u32x2 lo = *reinterpret_cast<const u32x2*>(tile + row * ld + col0 + 4 * half);
    u32x2 hi = *reinterpret_cast<const u32x2*>(tile + row * ld + col0 + 8 + 4 * half);
    u32x4 v = {lo.x, lo.y, hi.x, hi.y};
    return __builtin_bit_cast(bf16x8, v);
}

// B operand of the identity for the two k-steps of a 32-wide feature block
__device__ __forceinline__ void make_identity(int lane, bf16x8& i0, bf16x8& i1) {
    const int n = lane & 31, half = lane >> 5;
    u32x4 a, b;
    _Pragma("unroll") for (int w = 0; w < 4; ++w) {
        uint32_t va = 0, vb = 0;
        _Pragma("unroll") for (int s = 0; s < 2; ++s) {
            const int e = 2 * w + s, k = 8 * half + e;
            if (k == n) va |= 0x3f80u << (16 * s);
            if (16 + k == n) vb |= 0x3f80u << (16 * s);
        }
        a[w] = va;
        b[w] = vb;
    }
    i0 = __builtin_bit_cast(bf16x8, a);
    i1 = __builtin_bit_cast(bf16x8, b);
}

// D[m][n] = X[row0 + m][col0 + n] for a 32x32 block of a row-major LDS tile (exact: x * 1 in fp32)
__device__ __forceinline__ f32x16 turn_block(const uint16_t* tile, int ld, int row0, int col0, int lane,
                                             bf16x8 i0, bf16x8 i1) {
    const int m = lane & 31, half = lane >> 5;
    f32x16 acc = {0};
    acc = mfma(frag(tile, ld, row0 + m, col0 + 8 * half), i0, acc);
    acc = mfma(frag(tile, ld, row0 + m, col0 + 16 + 8 * half), i1, acc);
    return acc;
}

// registers 8*s .. 8*s+7 of a D-layout block as the operand of k-step s
__device__ __forceinline__ bf16x8 pack_step(const f32x16& d, int s) {
    u32x4 v = {pack2(d[8 * s + 0], d[8 * s + 1]), pack2(d[8 * s + 2], d[8 * s + 3]),
               pack2(d[8 * s + 4], d[8 * s + 5]), pack2(d[8 * s + 6], d[8 * s + 7])};
    return __builtin_bit_cast(bf16x8, v);
}

// write a D-layout block as 8-byte pieces: dst[(n)][m0 + 8g + 4half + 0..3], row stride ld
__device__ __forceinline__ void store_block_t(uint16_t* dst, int ld, int nrow, int m0, int half, const f32x16& d) {
    _Pragma("unroll") for (int g = 0; g < 4; ++g) {
        u32x2 v = {pack2(d[4 * g + 0], d[4 * g + 1]), pack2(d[4 * g + 2], d[4 * g + 3])};
        *reinterpret_cast<u32x2*>(dst + nrow * ld + m0 + 8 * g + 4 * half) = v;
    }
}

// same, as a bf16 head in `hi` and the bf16 remainder in `lo` (x = hi + lo to ~2^-17)
__device__ __forceinline__ void store_block_t_split(uint16_t* hi, uint16_t* lo, int ld, int nrow, int m0, int half,
                                                    const f32x16& d) {
    _Pragma("unroll") for (int g = 0; g < 4; ++g) {
        const uint32_t h0 = pack2(d[4 * g + 0], d[4 * g + 1]), h1 = pack2(d[4 * g + 2], d[4 * g + 3]);
        u32x2 vh = {h0, h1};
        u32x2 vl = {pack2(d[4 * g + 0] - bf16_lo(h0), d[4 * g + 1] - bf16_hi(h0)),
                    pack2(d[4 * g + 2] - bf16_lo(h1), d[4 * g + 3] - bf16_hi(h1))};
        *reinterpret_cast<u32x2*>(hi + nrow * ld + m0 + 8 * g + 4 * half) = vh;
        *reinterpret_cast<u32x2*>(lo + nrow * ld + m0 + 8 * g + 4 * half) = vl;
    }
}

// 64 x 128 bf16 tile: global rows [tok0, tok0+L) -> LDS (row stride LD), rows >= L zero
__device__ __forceinline__ void load_tile(uint16_t* dst, const uint16_t* src, size_t tok0, int L, int tid) {
    _Pragma("unroll") for (int it = 0; it < 4; ++it) {
        const int p = tid + kThreads * it, row = p >> 4, cp = p & 15;
        u32x4 v = {0, 0, 0, 0};
        if (row < L) v = *reinterpret_cast<const u32x4*>(src + (tok0 + row) * D + cp * 8);
        *reinterpret_cast<u32x4*>(dst + row * LD + cp * 8) = v;
    }
}
// LDS tile (row stride LD) rows [0, L) -> global
__device__ __forceinline__ void store_tile(uint16_t* dst, const uint16_t* src, size_t tok0, int L, int tid) {
    _Pragma("unroll") for (int it = 0; it < 4; ++it) {
        const int p = tid + kThreads * it, row = p >> 4, cp = p & 15;
        if (row < L)
            *reinterpret_cast<u32x4*>(dst + (tok0 + row) * D + cp * 8) =
                *reinterpret_cast<const u32x4*>(src + row * LD + cp * 8);
    }
}

// Chunk-local inclusive cumulative log-decay b_j, j = 0..63, into LDS (tokens >= L carry g = 0).
// Called by all threads; only wave 0 works.  Caller synchronises afterwards.
__device__ __forceinline__ void cumulative_decay(const Dims& d, const float* g, int bh, int t0, int L, float* bs,
                                                 int tid) {
    if (tid >= 64) return;
    float x = 0.f;
    if (tid < L) {
        if (d.kind == 1) x = g[bh % d.H];
        else if (d.kind == 2) x = g[size_t(bh) * d.T + t0 + tid];
    }
    for (int off = 1; off < 64; off <<= 1) {
        const float y = __shfl_up(x, off, 64);
        if (tid >= off) x += y;
    }
    bs[tid] = x;
}

// ---------------------------------------------------------------------------------------------
// Chunk states and the scan over chunks, fused: one wave owns a 32 x 32 block of the d_k x d_v
// state in MFMA accumulators (fp32) and walks the chunks of its sequence in order,
//     S_{c+1} = e^{b_C} S_c + sum_r (k_r e^{b_C - b_r})^T v_r ,
// writing the bf16 copy of S_c that the per-chunk kernels consume before each update.  The
// 16 waves of a (b,h) pair are independent (no LDS traffic between them, no barrier).
//   MODE 0: forward states, stored S^T [v][i]   (A side = k decayed, B side = v)
//   MODE 1: backward recomputation, stored S [i][v]   (A side = v, B side = k decayed)
//   MODE 2: reverse scan of state gradients, stored dS [i][v]: slot c receives the gradient of the
//           state at the END of chunk c;  dS_c = e^{b_C} dS_{c+1} + sum_j d_o_j^T (q_j e^{b_j})
//           (A side = d_o, B side = q decayed)
// Both operands of the token contraction come from identity turns, so their k order agrees.  The
// decayed operand is split into a bf16 head and a bf16 remainder (two MFMAs) so that the rounding of
// k * w does not show in a state that one token dominates.
// edge_in = M_0 (or d M_T), edge_out = M_T (or d M_0), fp32 [i][v], either may be NULL.
// states_rem (may be NULL) receives the bf16 remainder S - bf16(S) in the same layout: the decay
// gradient contracts q_u S d_o_u^T into one scalar per token, where the 2^-9 rounding of a state that
// a single token dominates is visible.
constexpr int kStatePrefetch = 2;
struct StateFrags {
    u32x4 a[4], b[4];  // [2*tb + s]: 8 features of token 32*tb + lane%32, A side and B side
    float g;
};

template <int MODE>
__device__ __forceinline__ void state_load(const Dims& d, const uint16_t* xa, const uint16_t* xb, const float* g,
                                           int bh, int c, int fa0, int fb0, int lane, StateFrags& f) {
    const int t0 = c * C, L = min(C, d.T - t0), m = lane & 31, half = lane >> 5;
    const size_t tok0 = size_t(bh) * d.T + t0;
    _Pragma("unroll") for (int tb = 0; tb < 2; ++tb) {
        const int tok = 32 * tb + m;
        _Pragma("unroll") for (int s = 0; s < 2; ++s) {
            u32x4 va = {0, 0, 0, 0}, vb = {0, 0, 0, 0};
            if (tok < L) {
                va = *reinterpret_cast<const u32x4*>(xa + (tok0 + tok) * D + fa0 + 16 * s + 8 * half);
                vb = *reinterpret_cast<const u32x4*>(xb + (tok0 + tok) * D + fb0 + 16 * s + 8 * half);
            }
            f.a[2 * tb + s] = va;
            f.b[2 * tb + s] = vb;
        }
    }
    f.g = 0.f;
    if (lane < L) {
        if (d.kind == 1) f.g = g[bh % d.H];
        else if (d.kind == 2) f.g = g[tok0 + lane];
    }
}

template <int MODE>
__global__ __launch_bounds__(kThreads) void mk_state_seq(Dims d, const uint16_t* __restrict__ xa,
                                                         const uint16_t* __restrict__ xb,
                                                         const float* __restrict__ g, uint16_t* __restrict__ states,
                                                         uint16_t* __restrict__ states_rem,
                                                         const float* __restrict__ edge_in,
                                                         float* __restrict__ edge_out) {
    __shared__ __align__(16) float wts[4][C];
    const int nb = blockIdx.x, bh = blockIdx.y, tid = threadIdx.x, lane = tid & 63, mb = tid >> 6;
    const int n = lane & 31, half = lane >> 5;
    constexpr bool kDecayA = MODE == 0;
    constexpr int sz = D * D;
    bf16x8 i0, i1;
    make_identity(lane, i0, i1);

    // acc[4g+j] = state element (m = 32mb + 8g + 4half + j, n = 32nb + lane%32); MODE 0: m = i, else m = v
    f32x16 acc = {0};
    if (edge_in) {
        const float* e = edge_in + size_t(bh) * sz;
        _Pragma("unroll") for (int r = 0; r < 16; ++r) {
            const int mm = 32 * mb + 8 * (r >> 2) + 4 * half + (r & 3), nn = 32 * nb + n;
            acc[r] = MODE == 0 ? e[mm * D + nn] : e[nn * D + mm];
        }
    }
    // loads run kStatePrefetch chunks ahead of the arithmetic: one chunk of arithmetic is shorter than
    // a trip to HBM, and each wave has nothing else to hide that latency with
    StateFrags fr[kStatePrefetch];
    const int first = MODE == 2 ? d.N - 1 : 0, step = MODE == 2 ? -1 : 1;
    _Pragma("unroll") for (int j = 0; j < kStatePrefetch; ++j)
        if (j < d.N) state_load<MODE>(d, xa, xb, g, bh, first + step * j, 32 * mb, 32 * nb, lane, fr[j]);
    for (int it0 = 0; it0 < d.N; it0 += kStatePrefetch) {
      _Pragma("unroll") for (int j = 0; j < kStatePrefetch; ++j) {
        const int it = it0 + j;
        if (it >= d.N) break;
        const int c = first + step * it;
        StateFrags& cur = fr[j];

        // emit the state this chunk starts from (MODE 2: the gradient this chunk ends with)
        uint16_t* dst = states + (size_t(bh) * d.N + c) * sz + (32 * nb + n) * D + 32 * mb + 4 * half;
        _Pragma("unroll") for (int gg = 0; gg < 4; ++gg) {
            u32x2 v = {pack2(acc[4 * gg], acc[4 * gg + 1]), pack2(acc[4 * gg + 2], acc[4 * gg + 3])};
            *reinterpret_cast<u32x2*>(dst + 8 * gg) = v;
            if (states_rem) {  // bf16 remainder of the same elements, for the consumer that needs ~16 bits
                u32x2 r = {pack2(acc[4 * gg] - bf16_lo(v.x), acc[4 * gg + 1] - bf16_hi(v.x)),
                           pack2(acc[4 * gg + 2] - bf16_lo(v.y), acc[4 * gg + 3] - bf16_hi(v.y))};
                *reinterpret_cast<u32x2*>(states_rem + (dst - states) + 8 * gg) = r;
            }
        }

        // chunk-local cumulative log-decay across the wave, per-token weight of the decayed operand
        float b = cur.g;
        for (int off = 1; off < 64; off <<= 1) {
            const float y = __shfl_up(b, off, 64);
            if (lane >= off) b += y;
        }
        const float bC = __shfl(b, 63, 64);
        const bool decays = d.kind != 0;
        if (decays) {
            __builtin_amdgcn_wave_barrier();
            wts[mb][lane] = MODE == 2 ? __expf(b) : __expf(bC - b);
            __builtin_amdgcn_wave_barrier();
        }
        bf16x8 A[4], B[4], R[4];  // R: remainder of the decayed side
        _Pragma("unroll") for (int tb = 0; tb < 2; ++tb) {
            f32x16 ta = {0}, tbk = {0};
            ta = mfma(__builtin_bit_cast(bf16x8, cur.a[2 * tb]), i0, ta);
            ta = mfma(__builtin_bit_cast(bf16x8, cur.a[2 * tb + 1]), i1, ta);
            tbk = mfma(__builtin_bit_cast(bf16x8, cur.b[2 * tb]), i0, tbk);
            tbk = mfma(__builtin_bit_cast(bf16x8, cur.b[2 * tb + 1]), i1, tbk);
            if (decays) {
                f32x16& t = kDecayA ? ta : tbk;
                f32x16 rem;
                _Pragma("unroll") for (int gg = 0; gg < 4; ++gg) {
                    const float4 w = *reinterpret_cast<const float4*>(&wts[mb][32 * tb + 8 * gg + 4 * half]);
                    t[4 * gg + 0] *= w.x; t[4 * gg + 1] *= w.y; t[4 * gg + 2] *= w.z; t[4 * gg + 3] *= w.w;
                }
                _Pragma("unroll") for (int r = 0; r < 16; r += 2) {
                    const uint32_t h = pack2(t[r], t[r + 1]);
                    rem[r] = t[r] - bf16_lo(h);
                    rem[r + 1] = t[r + 1] - bf16_hi(h);
                }
                R[2 * tb] = pack_step(rem, 0);
                R[2 * tb + 1] = pack_step(rem, 1);
            }
            A[2 * tb] = pack_step(ta, 0);
            A[2 * tb + 1] = pack_step(ta, 1);
            B[2 * tb] = pack_step(tbk, 0);
            B[2 * tb + 1] = pack_step(tbk, 1);
        }
        if (decays) {
            const float lamc = __expf(bC);
            _Pragma("unroll") for (int r = 0; r < 16; ++r) acc[r] *= lamc;
        }
        _Pragma("unroll") for (int ks = 0; ks < 4; ++ks) {
            acc = mfma(A[ks], B[ks], acc);
            if (decays) acc = kDecayA ? mfma(R[ks], B[ks], acc) : mfma(A[ks], R[ks], acc);
        }
        if (it + kStatePrefetch < d.N)
            state_load<MODE>(d, xa, xb, g, bh, c + step * kStatePrefetch, 32 * mb, 32 * nb, lane, cur);
      }
    }
    if (edge_out) {
        float* e = edge_out + size_t(bh) * sz;
        _Pragma("unroll") for (int r = 0; r < 16; ++r) {
            const int mm = 32 * mb + 8 * (r >> 2) + 4 * half + (r & 3), nn = 32 * nb + n;
            if (MODE == 0) e[mm * D + nn] = acc[r];
            else e[nn * D + mm] = acc[r];
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Output of one chunk:  O^T[v][j] = e^{b_j} sum_i S^T[v][i] q_j[i] + sum_{r<=j} V^T[v][r] P[j][r],
// P[j][r] = (q_j . k_r) e^{b_j - b_r}.   Wave w owns v in [32w, 32w+32).
// The scores are kept as a bf16 head and a bf16 remainder (two MFMAs per k-step): an output that one
// key dominates would otherwise carry the full 2^-9 rounding of its score.
// LDS: Q | K (later the O stage) | V (64 x LD each) | P head, P remainder (64 x LDP each) | bs
constexpr int kOutLds = (3 * C * LD + 2 * C * LDP) * 2 + C * 4;

__global__ __launch_bounds__(kThreads) void mk_output(Dims d, const uint16_t* __restrict__ q,
                                                      const uint16_t* __restrict__ k,
                                                      const uint16_t* __restrict__ v, const float* __restrict__ g,
                                                      const uint16_t* __restrict__ states,
                                                      uint16_t* __restrict__ o) {
    extern __shared__ __align__(16) unsigned char smem[];
    uint16_t* Q = reinterpret_cast<uint16_t*>(smem);
    uint16_t* K = Q + C * LD;
    uint16_t* V = K + C * LD;
    uint16_t* P = V + C * LD;
    uint16_t* Pr = P + C * LDP;
    float* bs = reinterpret_cast<float*>(Pr + C * LDP);
    uint16_t* stage = K;

    const int c = blockIdx.x, bh = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int t0 = c * C, L = min(C, d.T - t0);
    const size_t tok0 = size_t(bh) * d.T + t0;
    const int n = lane & 31, half = lane >> 5;

    // state rows of this wave straight from global memory: A operand [m = v][k = i]
    const uint16_t* St = states + (size_t(bh) * d.N + c) * D * D;
    bf16x8 sfrag[8];
    _Pragma("unroll") for (int ks = 0; ks < 8; ++ks)
        sfrag[ks] = *reinterpret_cast<const bf16x8*>(St + (32 * wave + n) * D + 16 * ks + 8 * half);

    load_tile(Q, q, tok0, L, tid);
    load_tile(K, k, tok0, L, tid);
    load_tile(V, v, tok0, L, tid);
    cumulative_decay(d, g, bh, t0, L, bs, tid);
    __syncthreads();

    // scores, quadrant (rb, jb) with rb <= jb:  D[m = r][n = j] = sum_i K[r][i] Q[j][i]
    {
        const int rb = wave & 1, jb = wave >> 1;
        if (rb <= jb) {
            f32x16 acc = {0};
            _Pragma("unroll") for (int ks = 0; ks < 8; ++ks)
                acc = mfma(frag(K, LD, 32 * rb + n, 16 * ks + 8 * half), frag(Q, LD, 32 * jb + n, 16 * ks + 8 * half), acc);
            const int j = 32 * jb + n;
            const float bj = bs[j];
            _Pragma("unroll") for (int r16 = 0; r16 < 16; ++r16) {
                const int r = 32 * rb + 8 * (r16 >> 2) + 4 * half + (r16 & 3);
                acc[r16] = r <= j ? acc[r16] * __expf(bj - bs[r]) : 0.f;
            }
            store_block_t_split(P, Pr, LDP, j, 32 * rb, half, acc);
        }
    }
    // V^T of this wave's 32 value columns, as A operand [m = v][k = r (permuted)]
    bf16x8 i0, i1;
    make_identity(lane, i0, i1);
    bf16x8 vt[4];
    _Pragma("unroll") for (int tb = 0; tb < 2; ++tb) {
        f32x16 t = turn_block(V, LD, 32 * tb, 32 * wave, lane, i0, i1);
        vt[2 * tb + 0] = pack_step(t, 0);
        vt[2 * tb + 1] = pack_step(t, 1);
    }
    __syncthreads();

    for (int jb = 0; jb < 2; ++jb) {
        f32x16 acc = {0};
        _Pragma("unroll") for (int ks = 0; ks < 8; ++ks) acc = mfma(sfrag[ks], frag(Q, LD, 32 * jb + n, 16 * ks + 8 * half), acc);
        const float w = __expf(bs[32 * jb + n]);
        _Pragma("unroll") for (int r = 0; r < 16; ++r) acc[r] *= w;
        const int kmax = jb == 0 ? 2 : 4;  // keys r >= 32 never reach queries j < 32
        _Pragma("unroll") for (int ks = 0; ks < 4; ++ks)
            if (ks < kmax) {
                acc = mfma(vt[ks], frag_perm(P, LDP, 32 * jb + n, 16 * ks, half), acc);
                acc = mfma(vt[ks], frag_perm(Pr, LDP, 32 * jb + n, 16 * ks, half), acc);
            }
        store_block_t(stage, LD, 32 * jb + n, 32 * wave, half, acc);
    }
    __syncthreads();
    store_tile(o, stage, tok0, L, tid);
}

// ---------------------------------------------------------------------------------------------
// Gradients of one chunk (scalar decay kinds).  S = state at the chunk start [i][v], dS = gradient
// of the state at the chunk end [i][v].  D_jr = e^{b_j-b_r} for r <= j, else 0.
//   dA = d_o V^T ,  G = dA * D ,  As = (Q K^T) * D
//   dq^T[i][j] = e^{b_j}     sum_v S[i][v]  d_o_j[v] + sum_r K^T[i][r] G[j][r]
//   dk^T[i][r] = e^{b_C-b_r} sum_v dS[i][v] v_r[v]   + sum_j Q^T[i][j] G[j][r]
//   dv^T[v][r] = e^{b_C-b_r} sum_i dS^T[v][i] k_r[i] + sum_j dO^T[v][j] As[j][r]
//   dg_t = sum_{u>=t} (q_u.dq_u - k_u.dk_u) + sum_r k_r.dk_r^{inter} + e^{b_C} <S, dS>
// Wave w owns i (and v) in [32w, 32w+32).
// G, its transpose and As are each kept as a bf16 head plus a bf16 remainder (see mk_output).
// LDS: Q | K | V | dO (64 x LD; later stages of dq, dk, dv) | G [j][r] | Gt [r][j] | Ast [r][j]
//      (head and remainder, 64 x LDP each) | bs (64) | red (4 x 64 x 3 floats: per-wave partial row dots) | zred
constexpr int kGradLds = (4 * C * LD + 6 * C * LDP) * 2 + C * 4 + 4 * 64 * 3 * 4 + 64;

__global__ __launch_bounds__(kThreads) void mk_grad(Dims d, const uint16_t* __restrict__ q,
                                                    const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
                                                    const uint16_t* __restrict__ d_o, const float* __restrict__ g,
                                                    const uint16_t* __restrict__ states,
                                                    const uint16_t* __restrict__ states_rem,
                                                    const uint16_t* __restrict__ dstates,
                                                    uint16_t* __restrict__ dq, uint16_t* __restrict__ dk,
                                                    uint16_t* __restrict__ dv, float* __restrict__ dg_tok) {
    extern __shared__ __align__(16) unsigned char smem[];
    uint16_t* Q = reinterpret_cast<uint16_t*>(smem);
    uint16_t* K = Q + C * LD;
    uint16_t* V = K + C * LD;
    uint16_t* dO = V + C * LD;
    constexpr int kRem = C * LDP;  // remainder tile follows its head
    uint16_t* G = dO + C * LD;
    uint16_t* Gt = G + 2 * C * LDP;
    uint16_t* Ast = Gt + 2 * C * LDP;
    float* bs = reinterpret_cast<float*>(Ast + 2 * C * LDP);
    float* red = bs + C;          // [wave][3][64]: q.dq, k.dk, k.dk_inter partial sums over this wave's i
    float* zred = red + 4 * 3 * 64;  // [wave]: partial <S, dS>

    const int c = blockIdx.x, bh = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int t0 = c * C, L = min(C, d.T - t0);
    const size_t tok0 = size_t(bh) * d.T + t0;
    const int n = lane & 31, half = lane >> 5;
    const uint16_t* S = states + (size_t(bh) * d.N + c) * D * D;
    const uint16_t* dS = dstates + (size_t(bh) * d.N + c) * D * D;

    // rows i in [32w, 32w+32) of S and dS: A operands [m = i][k = v]
    bf16x8 sfrag[8], dsfrag[8], srfrag[8];
    const bool want_dg = dg_tok != nullptr;  // then states_rem is present
    _Pragma("unroll") for (int ks = 0; ks < 8; ++ks) {
        sfrag[ks] = *reinterpret_cast<const bf16x8*>(S + (32 * wave + n) * D + 16 * ks + 8 * half);
        dsfrag[ks] = *reinterpret_cast<const bf16x8*>(dS + (32 * wave + n) * D + 16 * ks + 8 * half);
        if (want_dg)
            srfrag[ks] = *reinterpret_cast<const bf16x8*>(states_rem + (S - states) + (32 * wave + n) * D + 16 * ks +
                                                          8 * half);
    }
    load_tile(Q, q, tok0, L, tid);
    load_tile(K, k, tok0, L, tid);
    load_tile(V, v, tok0, L, tid);
    load_tile(dO, d_o, tok0, L, tid);
    cumulative_decay(d, g, bh, t0, L, bs, tid);
    __syncthreads();
    const float bC = bs[C - 1];

    // <S, dS> over this wave's rows
    if (dg_tok) {
        float z = 0.f;
        _Pragma("unroll") for (int ks = 0; ks < 8; ++ks) {
            u32x4 a = __builtin_bit_cast(u32x4, sfrag[ks]), b = __builtin_bit_cast(u32x4, dsfrag[ks]);
            u32x4 ar = __builtin_bit_cast(u32x4, srfrag[ks]);
            _Pragma("unroll") for (int p = 0; p < 4; ++p)
                z += (bf16_lo(a[p]) + bf16_lo(ar[p])) * bf16_lo(b[p]) + (bf16_hi(a[p]) + bf16_hi(ar[p])) * bf16_hi(b[p]);
        }
        for (int off = 32; off > 0; off >>= 1) z += __shfl_xor(z, off, 64);
        if (lane == 0) zred[wave] = z;
    }

    // score quadrants: 3 products x 3 non-zero quadrants = 9 jobs over 4 waves
    //   job kind 0: Ast[r][j] : D[m = j][n = r] = Q rows x K rows (k = i), masked and decayed
    //   job kind 1: G  [j][r] : D[m = r][n = j] = V rows x dO rows (k = v)
    //   job kind 2: Gt [r][j] : D[m = j][n = r] = dO rows x V rows
    for (int job = wave; job < 9; job += 4) {
        const int kind = job / 3, qd = job % 3;
        const int rb = qd == 2 ? 1 : 0, jb = qd == 0 ? 0 : 1;  // (0,0), (0,1), (1,1)
        const uint16_t* Am = kind == 0 ? Q : (kind == 1 ? V : dO);
        const uint16_t* Bm = kind == 0 ? K : (kind == 1 ? dO : V);
        const int mrow = kind == 1 ? 32 * rb : 32 * jb, nrow = kind == 1 ? 32 * jb : 32 * rb;
        f32x16 acc = {0};
        _Pragma("unroll") for (int ks = 0; ks < 8; ++ks)
            acc = mfma(frag(Am, LD, mrow + n, 16 * ks + 8 * half), frag(Bm, LD, nrow + n, 16 * ks + 8 * half), acc);
        _Pragma("unroll") for (int r16 = 0; r16 < 16; ++r16) {
            const int mi = mrow + 8 * (r16 >> 2) + 4 * half + (r16 & 3), ni = nrow + n;
            const int j = kind == 1 ? ni : mi, r = kind == 1 ? mi : ni;
            acc[r16] = r <= j ? acc[r16] * __expf(bs[j] - bs[r]) : 0.f;
        }
        uint16_t* dst = kind == 0 ? Ast : (kind == 1 ? G : Gt);
        store_block_t_split(dst, dst + kRem, LDP, nrow + n, mrow, half, acc);
    }
    bf16x8 i0, i1;
    make_identity(lane, i0, i1);
    __syncthreads();

    f32x16 accq[2], acck[2];
    // ---- dq^T[i][j] and dk^T[i][r] for i in this wave's slice
    {
        bf16x8 kt[4], qt[4];
        _Pragma("unroll") for (int tb = 0; tb < 2; ++tb) {
            f32x16 t = turn_block(K, LD, 32 * tb, 32 * wave, lane, i0, i1);
            kt[2 * tb] = pack_step(t, 0);
            kt[2 * tb + 1] = pack_step(t, 1);
            t = turn_block(Q, LD, 32 * tb, 32 * wave, lane, i0, i1);
            qt[2 * tb] = pack_step(t, 0);
            qt[2 * tb + 1] = pack_step(t, 1);
        }
        _Pragma("unroll") for (int nb = 0; nb < 2; ++nb) {
            const int tok = 32 * nb + n;  // j for dq, r for dk
            f32x16 aq = {0}, ak = {0}, aqr = {0};  // aqr: remainder of S, enters the decay gradient only
            _Pragma("unroll") for (int ks = 0; ks < 8; ++ks) {
                const bf16x8 dof = frag(dO, LD, tok, 16 * ks + 8 * half);
                aq = mfma(sfrag[ks], dof, aq);
                if (want_dg) aqr = mfma(srfrag[ks], dof, aqr);
                ak = mfma(dsfrag[ks], frag(V, LD, tok, 16 * ks + 8 * half), ak);
            }
            const float wq = __expf(bs[tok]), wk = __expf(bC - bs[tok]);
            float pk_inter = 0.f;
            _Pragma("unroll") for (int r = 0; r < 16; ++r) { aq[r] *= wq; ak[r] *= wk; }
            if (want_dg) {
                // k . dk_inter over this lane's 16 features
                _Pragma("unroll") for (int gg = 0; gg < 4; ++gg) {
                    u32x2 kk = *reinterpret_cast<const u32x2*>(K + tok * LD + 32 * wave + 8 * gg + 4 * half);
                    pk_inter += bf16_lo(kk.x) * ak[4 * gg] + bf16_hi(kk.x) * ak[4 * gg + 1] +
                                bf16_lo(kk.y) * ak[4 * gg + 2] + bf16_hi(kk.y) * ak[4 * gg + 3];
                }
            }
            // intra: dq over keys r <= j (k-steps of r), dk over queries j >= r (k-steps of j)
            _Pragma("unroll") for (int ks = 0; ks < 4; ++ks) {
                if (!(nb == 0 && ks >= 2)) {
                    aq = mfma(kt[ks], frag_perm(G, LDP, tok, 16 * ks, half), aq);
                    aq = mfma(kt[ks], frag_perm(G + kRem, LDP, tok, 16 * ks, half), aq);
                }
                if (!(nb == 1 && ks < 2)) {
                    ak = mfma(qt[ks], frag_perm(Gt, LDP, tok, 16 * ks, half), ak);
                    ak = mfma(qt[ks], frag_perm(Gt + kRem, LDP, tok, 16 * ks, half), ak);
                }
            }
            accq[nb] = aq;
            acck[nb] = ak;
            if (want_dg) {
                float pq = 0.f, pk = 0.f;
                _Pragma("unroll") for (int gg = 0; gg < 4; ++gg) {
                    u32x2 qq = *reinterpret_cast<const u32x2*>(Q + tok * LD + 32 * wave + 8 * gg + 4 * half);
                    u32x2 kk = *reinterpret_cast<const u32x2*>(K + tok * LD + 32 * wave + 8 * gg + 4 * half);
                    pq += bf16_lo(qq.x) * (aq[4 * gg] + wq * aqr[4 * gg]) + bf16_hi(qq.x) * (aq[4 * gg + 1] + wq * aqr[4 * gg + 1]) +
                          bf16_lo(qq.y) * (aq[4 * gg + 2] + wq * aqr[4 * gg + 2]) + bf16_hi(qq.y) * (aq[4 * gg + 3] + wq * aqr[4 * gg + 3]);
                    pk += bf16_lo(kk.x) * ak[4 * gg] + bf16_hi(kk.x) * ak[4 * gg + 1] + bf16_lo(kk.y) * ak[4 * gg + 2] +
                          bf16_hi(kk.y) * ak[4 * gg + 3];
                }
                pq += __shfl_xor(pq, 32, 64);
                pk += __shfl_xor(pk, 32, 64);
                pk_inter += __shfl_xor(pk_inter, 32, 64);
                if (half == 0) {
                    red[(wave * 3 + 0) * 64 + tok] = pq;
                    red[(wave * 3 + 1) * 64 + tok] = pk;
                    red[(wave * 3 + 2) * 64 + tok] = pk_inter;
                }
            }
        }
    }
    // ---- dv^T[v][r] for v in this wave's slice
    f32x16 accv[2];
    {
        // dS^T rows of this wave: turn dS[i-block][v-slice] straight from global memory
        bf16x8 dst_[8], dot[4];
        const int m = lane & 31;
        _Pragma("unroll") for (int ib = 0; ib < 4; ++ib) {
            f32x16 t = {0};
            t = mfma(*reinterpret_cast<const bf16x8*>(dS + (32 * ib + m) * D + 32 * wave + 8 * half), i0, t);
            t = mfma(*reinterpret_cast<const bf16x8*>(dS + (32 * ib + m) * D + 32 * wave + 16 + 8 * half), i1, t);
            dst_[2 * ib] = pack_step(t, 0);
            dst_[2 * ib + 1] = pack_step(t, 1);
        }
        _Pragma("unroll") for (int tb = 0; tb < 2; ++tb) {
            f32x16 t = turn_block(dO, LD, 32 * tb, 32 * wave, lane, i0, i1);
            dot[2 * tb] = pack_step(t, 0);
            dot[2 * tb + 1] = pack_step(t, 1);
        }
        _Pragma("unroll") for (int nb = 0; nb < 2; ++nb) {
            const int r = 32 * nb + n;
            f32x16 av = {0};
            _Pragma("unroll") for (int ks = 0; ks < 8; ++ks) av = mfma(dst_[ks], frag_perm(K, LD, r, 16 * ks, half), av);
            const float wk = __expf(bC - bs[r]);
            _Pragma("unroll") for (int x = 0; x < 16; ++x) av[x] *= wk;
            _Pragma("unroll") for (int ks = 0; ks < 4; ++ks)
                if (!(nb == 1 && ks < 2)) {
                    av = mfma(dot[ks], frag_perm(Ast, LDP, r, 16 * ks, half), av);
                    av = mfma(dot[ks], frag_perm(Ast + kRem, LDP, r, 16 * ks, half), av);
                }
            accv[nb] = av;
        }
    }
    __syncthreads();  // every wave is done with Q, K, V, dO, G, Gt, Ast
    _Pragma("unroll") for (int nb = 0; nb < 2; ++nb) {
        store_block_t(Q, LD, 32 * nb + n, 32 * wave, half, accq[nb]);
        store_block_t(K, LD, 32 * nb + n, 32 * wave, half, acck[nb]);
        store_block_t(V, LD, 32 * nb + n, 32 * wave, half, accv[nb]);
    }
    __syncthreads();
    store_tile(dq, Q, tok0, L, tid);
    store_tile(dk, K, tok0, L, tid);
    store_tile(dv, V, tok0, L, tid);
    if (want_dg && tid < 64) {
        // fixed-order sums over the four feature slices, then the reverse in-chunk running sum
        float w = 0.f, tail = 0.f, z = (zred[0] + zred[1]) + (zred[2] + zred[3]);
        _Pragma("unroll") for (int wv = 0; wv < 4; ++wv) {
            w += red[(wv * 3 + 0) * 64 + tid] - red[(wv * 3 + 1) * 64 + tid];
            tail += red[(wv * 3 + 2) * 64 + tid];
        }
        for (int off = 32; off > 0; off >>= 1) tail += __shfl_xor(tail, off, 64);
        // suffix sum of w over tokens >= tid
        float sfx = w;
        for (int off = 1; off < 64; off <<= 1) {
            const float y = __shfl_down(sfx, off, 64);
            if (tid + off < 64) sfx += y;
        }
        if (tid < L) dg_tok[tok0 + tid] = sfx + tail + __expf(bC) * z;
    }
}

// dg[h] = sum_{b,t} dg_tok[b,h,t] in a fixed order (grid: H)
__global__ void mk_head_reduce(Dims d, const float* __restrict__ dg_tok, float* __restrict__ dg) {
    __shared__ float part[kThreads];
    const int h = blockIdx.x;
    float s = 0.f;
    const size_t nn = size_t(d.B) * d.T;
    for (size_t e = threadIdx.x; e < nn; e += blockDim.x) s += dg_tok[((e / d.T) * d.H + h) * d.T + e % d.T];
    part[threadIdx.x] = s;
    __syncthreads();
    for (int w = kThreads / 2; w > 0; w >>= 1) {
        if (threadIdx.x < w) part[threadIdx.x] += part[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) dg[h] = part[0];
}

struct Ws {
    uint16_t *states, *dstates, *states_rem;
    float* dg_tok;
    size_t bytes;
};

Ws carve(const Dims& d, void* ws, bool bwd) {
    char* p = static_cast<char*>(ws);
    size_t off = 0;
    Ws w{};
    const size_t st = align256(size_t(d.BH()) * d.N * D * D * 2);
    w.states = reinterpret_cast<uint16_t*>(p + off); off += st;
    if (bwd) { w.dstates = reinterpret_cast<uint16_t*>(p + off); off += st; }
    if (bwd && d.kind != 0) { w.states_rem = reinterpret_cast<uint16_t*>(p + off); off += st; }
    if (bwd && d.kind == 1) { w.dg_tok = reinterpret_cast<float*>(p + off); off += align256(size_t(d.BH()) * d.T * 4); }
    w.bytes = off;
    return w;
}

template <typename K>
hipError_t allow_lds(K kernel, int bytes) {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
}

}  // namespace

bool mfma_supported(const Dims& d) {
    return d.bf16 && d.C == C && d.dk == D && d.dv == D && d.kind != 3;
}

size_t mfma_fwd_workspace(const Dims& d) { return carve(d, nullptr, false).bytes; }
size_t mfma_bwd_workspace(const Dims& d) { return carve(d, nullptr, true).bytes; }

hipError_t mfma_fwd(const Dims& d, const FwdArgs& a) {
    Ws w = carve(d, a.ws, false);
    const dim3 grid(d.N, d.BH()), block(kThreads), sgrid(D / 32, d.BH());
    auto q = static_cast<const uint16_t*>(a.q), k = static_cast<const uint16_t*>(a.k), v = static_cast<const uint16_t*>(a.v);
    hipError_t e;
    if ((e = allow_lds(mk_output, kOutLds)) != hipSuccess) return e;
    { ProfScope ps(KID_MFMA_STATE, a.stream); hipLaunchKernelGGL((mk_state_seq<0>), sgrid, block, 0, a.stream, d, k, v, a.g, w.states,
                       static_cast<uint16_t*>(nullptr), a.m0, a.mT); }
    { ProfScope ps(KID_MFMA_OUTPUT, a.stream); hipLaunchKernelGGL(mk_output, grid, block, kOutLds, a.stream, d, q, k, v, a.g, w.states,
                       static_cast<uint16_t*>(a.o)); }
    return hipGetLastError();
}

hipError_t mfma_bwd(const Dims& d, const BwdArgs& a) {
    Ws w = carve(d, a.ws, true);
    const dim3 grid(d.N, d.BH()), block(kThreads), sgrid(D / 32, d.BH());
    auto q = static_cast<const uint16_t*>(a.q), k = static_cast<const uint16_t*>(a.k), v = static_cast<const uint16_t*>(a.v);
    auto d_o = static_cast<const uint16_t*>(a.d_o);
    hipError_t e;
    if ((e = allow_lds(mk_grad, kGradLds)) != hipSuccess) return e;
    { ProfScope ps(KID_MFMA_STATE_BWD, a.stream); hipLaunchKernelGGL((mk_state_seq<1>), sgrid, block, 0, a.stream, d, v, k, a.g, w.states,
                       a.dg ? w.states_rem : static_cast<uint16_t*>(nullptr), a.m0, static_cast<float*>(nullptr)); }
    { ProfScope ps(KID_MFMA_DSTATE, a.stream); hipLaunchKernelGGL((mk_state_seq<2>), sgrid, block, 0, a.stream, d, d_o, q, a.g, w.dstates,
                       static_cast<uint16_t*>(nullptr), a.d_mT, a.d_m0); }
    float* dg_tok = nullptr;
    if (a.dg) dg_tok = d.kind == 1 ? w.dg_tok : a.dg;  // per-token scalar decay: written in place
    { ProfScope ps(KID_MFMA_GRAD, a.stream); hipLaunchKernelGGL(mk_grad, grid, block, kGradLds, a.stream, d, q, k, v, d_o, a.g, w.states, w.states_rem, w.dstates,
                       static_cast<uint16_t*>(a.dq), static_cast<uint16_t*>(a.dk), static_cast<uint16_t*>(a.dv), dg_tok); }
    if (a.dg && d.kind == 1) {
        ProfScope ps(KID_HEAD_REDUCE, a.stream);
        hipLaunchKernelGGL(mk_head_reduce, dim3(d.H), block, 0, a.stream, d, w.dg_tok, a.dg);
    }
    return hipGetLastError();
}

}  // namespace lsm
