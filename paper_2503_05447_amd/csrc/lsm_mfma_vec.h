// MFMA kernels for the per-key-feature (vector) decay kind: a_t in R^{d_k} (Table 1, GLA / RWKV6 /
// HGRN2 rows), bf16 operands, chunk = 64, d_k = 128, d_v a multiple of 128.  Included by lsm_mfma.hip.
//
// With a decay per feature the intra-chunk score no longer factors into (q.k) times one weight:
//     P[j][r] = sum_i q_j[i] k_r[i] e^{b_j[i] - b_r[i]} ,  r <= j .
// Splitting the exponent at a reference token m with r < m <= j gives two factors that are both <= 1,
//     e^{b_j - b_{m-1}}  (query side)   and   e^{b_{m-1} - b_r}  (key side),
// so the weighted operands can be rounded to bf16 and contracted on the matrix cores without overflow
// for any decay strength (splitting at the chunk start instead would need e^{-b_r}, which overflows).
// The reference must lie between r and j, so the 64 x 64 triangle is covered level by level: at level
// s = 32, 16, 8, 4, 2, 1 the pairs whose token indices first differ in bit log2(s) are handled together:
// j lies in an odd block of s tokens, r in the even block before it, m = the start of j's block.  At
// every level each token is on exactly one side, so one 64 x 128 tile W_s (row t = q_t or k_t times its
// weight) serves as both operands: the level's scores are entries of the Gram matrix W_s W_s^T.  The
// diagonal r = j carries no decay and is an exact dot product.
#pragma once

constexpr int LDF = D + 4;  // row stride (floats) of the fp32 [64][128] cumulative-decay tile in LDS

// log2 of the level s at which the pair (a, b) of chunk-local token indices is handled; a != b
__device__ __forceinline__ int pair_level(int a, int b) { return 31 - __clz(a ^ b); }

// weight exponent of token t at level s = 1 << ls:  q side (odd block): b_t - b_{m-1};  k side: b_{e} - b_t
// with e the last token of t's own block.  Returns the reference row and sets `qside`.
__device__ __forceinline__ int level_ref(int t, int ls, bool& qside) {
    const int blk = t >> ls;
    qside = blk & 1;
    return qside ? (blk << ls) - 1 : (blk << ls) + (1 << ls) - 1;
}

// exp of 8 differences, applied to 8 bf16 values (packed in u32x4), result as bf16 head (+ remainder)
__device__ __forceinline__ void weigh8(const u32x4& raw, const float* w, u32x4& hi, u32x4* lo) {
    _Pragma("unroll") for (int p = 0; p < 4; ++p) {
        const float x0 = bf16_lo(raw[p]) * w[2 * p], x1 = bf16_hi(raw[p]) * w[2 * p + 1];
        const uint32_t h = pack2(x0, x1);
        hi[p] = h;
        if (lo) (*lo)[p] = pack2(x0 - bf16_lo(h), x1 - bf16_hi(h));
    }
}

// ---------------------------------------------------------------------------------------------
// Per chunk (grid: N x BH): cumulative log-decay b [64][128]; the decayed operands of the state
// passes  khat = k e^{b_C - b},  qhat = q e^{b}  as bf16 head and remainder planes [BH*T][128];
// lam = e^{b_C} [BH*N][128];  and the masked decayed scores P [BH*N][64][64] (head, remainder).
// W_s is kept as a bf16 head and a bf16 remainder (three MFMAs per step: hh + hl + lh): with single
// bf16 operands the 2^-9 rounding of every weighted element, summed over 128 features and 64 keys,
// already takes half of the error budget of o.
// LDS: b tile (fp32) | W head | W remainder; after the last level the same memory holds the waves'
// partial score blocks for the final sum.
constexpr int kPrepRedLd = 36;                                  // row stride (floats) of a 32 x 32 partial block
constexpr int kPrepLdsMain = C * LDF * 4 + 2 * C * LD * 2;      // 68.6 KB
constexpr int kPrepLdsRed = 8 * 32 * kPrepRedLd * 4;            // 36.9 KB (aliases the main area)
constexpr int kPrepLds = kPrepLdsMain + C * 4;                  // + diagonal dots

__global__ __launch_bounds__(kThreads, 2) void mk_vec_prep(Dims d, const uint16_t* __restrict__ q,
                                                           const uint16_t* __restrict__ k, const float* __restrict__ g,
                                                           uint16_t* __restrict__ khat_hi, uint16_t* __restrict__ khat_lo,
                                                           uint16_t* __restrict__ qhat_hi, uint16_t* __restrict__ qhat_lo,
                                                           float* __restrict__ lamv, uint16_t* __restrict__ p_hi,
                                                           uint16_t* __restrict__ p_lo) {
    extern __shared__ __align__(16) unsigned char smem[];
    float* bt = reinterpret_cast<float*>(smem);                       // [64][LDF]
    uint16_t* Wh = reinterpret_cast<uint16_t*>(bt + C * LDF);         // [64][LD] head
    uint16_t* Wl = Wh + C * LD;                                       // [64][LD] remainder
    float* red = reinterpret_cast<float*>(smem);                      // [8][32][kPrepRedLd], after the levels
    float* diag = reinterpret_cast<float*>(smem + kPrepLdsMain);      // [64]

    const int c = blockIdx.x, bh = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int t0 = c * C, L = min(C, d.T - t0);
    const size_t tok0 = size_t(bh) * d.T + t0;
    const int n = lane & 31, half = lane >> 5;
    const int cp = tid & 15, r0 = tid >> 4;  // this thread's feature piece (8 features) and first row; rows r0 + 16 it

    // raw q, k pieces stay in registers for all levels; g goes to LDS for the scan along tokens
    u32x4 qr[4], kr[4];
    _Pragma("unroll") for (int it = 0; it < 4; ++it) {
        const int row = r0 + 16 * it;
        float4 g0 = {0.f, 0.f, 0.f, 0.f}, g1 = g0;
        qr[it] = u32x4{0, 0, 0, 0};
        kr[it] = u32x4{0, 0, 0, 0};
        if (row < L) {
            qr[it] = *reinterpret_cast<const u32x4*>(q + (tok0 + row) * D + cp * 8);
            kr[it] = *reinterpret_cast<const u32x4*>(k + (tok0 + row) * D + cp * 8);
            g0 = *reinterpret_cast<const float4*>(g + (tok0 + row) * D + cp * 8);
            g1 = *reinterpret_cast<const float4*>(g + (tok0 + row) * D + cp * 8 + 4);
        }
        *reinterpret_cast<float4*>(bt + row * LDF + cp * 8) = g0;
        *reinterpret_cast<float4*>(bt + row * LDF + cp * 8 + 4) = g1;
    }
    // diagonal scores q_t . k_t: exact products, summed over this thread's 8 features, then over the
    // 16 threads that share the row (consecutive lanes)
    _Pragma("unroll") for (int it = 0; it < 4; ++it) {
        float s = 0.f;
        _Pragma("unroll") for (int p = 0; p < 4; ++p)
            s += bf16_lo(qr[it][p]) * bf16_lo(kr[it][p]) + bf16_hi(qr[it][p]) * bf16_hi(kr[it][p]);
        _Pragma("unroll") for (int off = 8; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
        if (cp == 0) diag[r0 + 16 * it] = s;
    }
    __syncthreads();
    {   // inclusive scan along tokens, one feature column per thread, two halves of 32 tokens
        const int i = tid & 127, hh = tid >> 7;
        float run = 0.f;
        for (int r = 32 * hh; r < 32 * hh + 32; ++r) {
            run += bt[r * LDF + i];
            bt[r * LDF + i] = run;
        }
        __syncthreads();
        if (hh == 1) {
            const float base = bt[31 * LDF + i];
            for (int r = 32; r < 64; ++r) bt[r * LDF + i] += base;
        }
    }
    __syncthreads();
    float bC[8];
    {
        const float4 x0 = *reinterpret_cast<const float4*>(bt + 63 * LDF + cp * 8);
        const float4 x1 = *reinterpret_cast<const float4*>(bt + 63 * LDF + cp * 8 + 4);
        bC[0] = x0.x; bC[1] = x0.y; bC[2] = x0.z; bC[3] = x0.w; bC[4] = x1.x; bC[5] = x1.y; bC[6] = x1.z; bC[7] = x1.w;
    }
    auto brow = [&](int row, float* out) {
        const float4 x0 = *reinterpret_cast<const float4*>(bt + row * LDF + cp * 8);
        const float4 x1 = *reinterpret_cast<const float4*>(bt + row * LDF + cp * 8 + 4);
        out[0] = x0.x; out[1] = x0.y; out[2] = x0.z; out[3] = x0.w; out[4] = x1.x; out[5] = x1.y; out[6] = x1.z; out[7] = x1.w;
    };
    // decayed operands of the state passes
    _Pragma("unroll") for (int it = 0; it < 4; ++it) {
        const int row = r0 + 16 * it;
        float b[8], wk[8], wq[8];
        brow(row, b);
        _Pragma("unroll") for (int e = 0; e < 8; ++e) {
            wk[e] = __expf(bC[e] - b[e]);
            wq[e] = __expf(b[e]);
        }
        u32x4 hi, lo;
        if (row < L) {
            weigh8(kr[it], wk, hi, &lo);
            *reinterpret_cast<u32x4*>(khat_hi + (tok0 + row) * D + cp * 8) = hi;
            *reinterpret_cast<u32x4*>(khat_lo + (tok0 + row) * D + cp * 8) = lo;
            weigh8(qr[it], wq, hi, &lo);
            *reinterpret_cast<u32x4*>(qhat_hi + (tok0 + row) * D + cp * 8) = hi;
            *reinterpret_cast<u32x4*>(qhat_lo + (tok0 + row) * D + cp * 8) = lo;
        }
    }
    if (tid < D) lamv[(size_t(bh) * d.N + c) * D + tid] = __expf(bt[63 * LDF + tid]);

    // levels: wave w accumulates, masked, the partial Gram blocks it is responsible for
    //   accD: diagonal 32-block (w & 1), feature range 64 (w >> 1) .. + 64     (levels 16 .. 1)
    //   accO: block (keys 0..31, queries 32..63), feature range 32 w .. + 32   (level 32)
    f32x16 accD = {0}, accO = {0};
    _Pragma("unroll") for (int lv = 0; lv < 6; ++lv) {
        const int ls = 5 - lv;
        if (lv > 0) __syncthreads();  // every wave has read the previous level's tiles
        _Pragma("unroll") for (int it = 0; it < 4; ++it) {
            const int row = r0 + 16 * it;
            bool qside;
            const int ref = level_ref(row, ls, qside);
            float b[8], br[8], w[8];
            brow(row, b);
            brow(ref, br);
            _Pragma("unroll") for (int e = 0; e < 8; ++e) w[e] = __expf(qside ? b[e] - br[e] : br[e] - b[e]);
            u32x4 hi, lo;
            weigh8(qside ? qr[it] : kr[it], w, hi, &lo);
            *reinterpret_cast<u32x4*>(Wh + row * LD + cp * 8) = hi;
            *reinterpret_cast<u32x4*>(Wl + row * LD + cp * 8) = lo;
        }
        __syncthreads();  // W of this level complete
        if (ls == 5) {
            _Pragma("unroll") for (int s2 = 0; s2 < 2; ++s2) {
                const int col = 16 * (2 * wave + s2) + 8 * half;
                const bf16x8 ah = frag(Wh, LD, n, col), al = frag(Wl, LD, n, col);
                const bf16x8 bh = frag(Wh, LD, 32 + n, col), bl = frag(Wl, LD, 32 + n, col);
                accO = mfma(ah, bh, accO);  // D[m = r][n = j - 32]
                accO = mfma(ah, bl, accO);
                accO = mfma(al, bh, accO);
            }
        } else {
            f32x16 lev = {0};
            const int blk = wave & 1;
            _Pragma("unroll") for (int s4 = 0; s4 < 4; ++s4) {
                const int col = 16 * (4 * (wave >> 1) + s4) + 8 * half;
                const bf16x8 fh = frag(Wh, LD, 32 * blk + n, col), fl = frag(Wl, LD, 32 * blk + n, col);
                lev = mfma(fh, fh, lev);  // Gram block: D[m][n] = W_m . W_n
                lev = mfma(fh, fl, lev);
                lev = mfma(fl, fh, lev);
            }
            _Pragma("unroll") for (int x = 0; x < 16; ++x) {
                const int m = 8 * (x >> 2) + 4 * half + (x & 3);
                const bool valid = ((m ^ n) >> ls) == 1 && ((n >> ls) & 1);  // r = m in the even block, j = n in the odd
                accD[x] += valid ? lev[x] : 0.f;
            }
        }
    }
    __syncthreads();  // all reads of b and W done: the memory becomes the reduction area
    {
        float* rd = red + wave * 32 * kPrepRedLd;        // [n = j][m = r]
        float* ro = red + (4 + wave) * 32 * kPrepRedLd;
        _Pragma("unroll") for (int gq = 0; gq < 4; ++gq) {
            *reinterpret_cast<float4*>(rd + n * kPrepRedLd + 8 * gq + 4 * half) =
                float4{accD[4 * gq], accD[4 * gq + 1], accD[4 * gq + 2], accD[4 * gq + 3]};
            *reinterpret_cast<float4*>(ro + n * kPrepRedLd + 8 * gq + 4 * half) =
                float4{accO[4 * gq], accO[4 * gq + 1], accO[4 * gq + 2], accO[4 * gq + 3]};
        }
    }
    __syncthreads();
    {   // P[j][r0 .. r0+15]: fixed-order sum of the partial blocks, diagonal, split, store
        const int j = tid >> 2, rbase = 16 * (tid & 3);
        const int jb = j >> 5, rb = rbase >> 5, jn = j & 31, rm = rbase & 31;
        float val[16];
        _Pragma("unroll") for (int e = 0; e < 16; ++e) val[e] = 0.f;
        if (rb == jb) {
            const float* a = red + jb * 32 * kPrepRedLd + jn * kPrepRedLd + rm;
            const float* b = red + (jb + 2) * 32 * kPrepRedLd + jn * kPrepRedLd + rm;
            _Pragma("unroll") for (int e = 0; e < 16; ++e) val[e] = a[e] + b[e];
            if ((j >> 4) == (rbase >> 4)) {
                const float dj = diag[j];
                _Pragma("unroll") for (int e = 0; e < 16; ++e) val[e] = (rbase + e == j) ? dj : val[e];
            }
        } else if (rb < jb) {
            const float* a = red + 4 * 32 * kPrepRedLd + jn * kPrepRedLd + rm;
            _Pragma("unroll") for (int e = 0; e < 16; ++e)
                val[e] = (a[e] + a[e + 32 * kPrepRedLd]) + (a[e + 64 * kPrepRedLd] + a[e + 96 * kPrepRedLd]);
        }
        u32x4 hi[2], lo[2];
        _Pragma("unroll") for (int p = 0; p < 8; ++p) {
            const uint32_t h = pack2(val[2 * p], val[2 * p + 1]);
            hi[p >> 2][p & 3] = h;
            lo[p >> 2][p & 3] = pack2(val[2 * p] - bf16_lo(h), val[2 * p + 1] - bf16_hi(h));
        }
        const size_t off = (size_t(bh) * d.N + c) * C * C + j * C + rbase;
        *reinterpret_cast<u32x4*>(p_hi + off) = hi[0];
        *reinterpret_cast<u32x4*>(p_hi + off + 8) = hi[1];
        *reinterpret_cast<u32x4*>(p_lo + off) = lo[0];
        *reinterpret_cast<u32x4*>(p_lo + off + 8) = lo[1];
    }
}

// 64 x 128 bf16 tile out of rows of `stride` elements starting at column `col0`; rows >= L zero
__device__ __forceinline__ void load_tile_strided(uint16_t* dst, const uint16_t* src, size_t tok0, int L, int stride,
                                                  int col0, int tid) {
    _Pragma("unroll") for (int it = 0; it < 4; ++it) {
        const int p = tid + kThreads * it, row = p >> 4, cp = p & 15;
        u32x4 v = {0, 0, 0, 0};
        if (row < L) v = *reinterpret_cast<const u32x4*>(src + (tok0 + row) * stride + col0 + cp * 8);
        *reinterpret_cast<u32x4*>(dst + row * LD + cp * 8) = v;
    }
}
__device__ __forceinline__ void store_tile_strided(uint16_t* dst, const uint16_t* src, size_t tok0, int L, int stride,
                                                   int col0, int tid) {
    _Pragma("unroll") for (int it = 0; it < 4; ++it) {
        const int p = tid + kThreads * it, row = p >> 4, cp = p & 15;
        if (row < L)
            *reinterpret_cast<u32x4*>(dst + (tok0 + row) * stride + col0 + cp * 8) =
                *reinterpret_cast<const u32x4*>(src + row * LD + cp * 8);
    }
}
// 64 x 64 bf16 matrix (dense rows) -> LDS tile with row stride LDP
__device__ __forceinline__ void load_scores(uint16_t* dst, const uint16_t* src, int tid) {
    _Pragma("unroll") for (int it = 0; it < 2; ++it) {
        const int p = tid + kThreads * it, row = p >> 3, cp = p & 7;
        *reinterpret_cast<u32x4*>(dst + row * LDP + cp * 8) = *reinterpret_cast<const u32x4*>(src + row * C + cp * 8);
    }
}

// ---------------------------------------------------------------------------------------------
// Output of one chunk for one 128-wide slice of the value dimension (grid: N x BH x d_v/128):
//   O^T[v][j] = sum_i S^T[v][i] qhat_j[i] + sum_{r<=j} V^T[v][r] P[j][r]
// with qhat and P from mk_vec_prep.  Wave w owns 32 value columns.
// LDS: qhat head (later the O stage) | qhat remainder | V slice | P head | P remainder
constexpr int kOutVecLds = 3 * C * LD * 2 + 2 * C * LDP * 2;

__global__ __launch_bounds__(kThreads, 2) void mk_output_vec(Dims d, const uint16_t* __restrict__ qhat,
                                                             const uint16_t* __restrict__ qhat_lo,
                                                             const uint16_t* __restrict__ v,
                                                             const uint16_t* __restrict__ p_hi,
                                                             const uint16_t* __restrict__ p_lo,
                                                             const uint16_t* __restrict__ states,
                                                             uint16_t* __restrict__ o) {
    extern __shared__ __align__(16) unsigned char smem[];
    uint16_t* Q = reinterpret_cast<uint16_t*>(smem);
    uint16_t* Ql = Q + C * LD;
    uint16_t* V = Ql + C * LD;
    uint16_t* Ph = V + C * LD;
    uint16_t* Pl = Ph + C * LDP;

    const int c = blockIdx.x, bh = blockIdx.y, vh = blockIdx.z, nvh = gridDim.z;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int t0 = c * C, L = min(C, d.T - t0);
    const size_t tok0 = size_t(bh) * d.T + t0;
    const int n = lane & 31, half = lane >> 5;

    const uint16_t* St = states + ((size_t(bh) * nvh + vh) * d.N + c) * D * D;
    bf16x8 sfrag[8];
    _Pragma("unroll") for (int ks = 0; ks < 8; ++ks)
        sfrag[ks] = *reinterpret_cast<const bf16x8*>(St + (32 * wave + n) * D + 16 * ks + 8 * half);

    load_tile(Q, qhat, tok0, L, tid);
    load_tile(Ql, qhat_lo, tok0, L, tid);
    load_tile_strided(V, v, tok0, L, d.dv, D * vh, tid);
    const size_t poff = (size_t(bh) * d.N + c) * C * C;
    load_scores(Ph, p_hi + poff, tid);
    load_scores(Pl, p_lo + poff, tid);
    __syncthreads();

    PackedBlock res[2];
    _Pragma("unroll") for (int jb = 0; jb < 2; ++jb) {
        const int j = 32 * jb + n;
        f32x16 acc = {0};
        _Pragma("unroll") for (int ks = 0; ks < 8; ++ks) {
            acc = mfma(sfrag[ks], frag(Q, LD, j, 16 * ks + 8 * half), acc);
            acc = mfma(sfrag[ks], frag(Ql, LD, j, 16 * ks + 8 * half), acc);
        }
        _Pragma("unroll") for (int ks = 0; ks < 2 * (jb + 1); ++ks) {  // keys r >= 32 never reach queries j < 32
            const bf16x8 vt = frag_tr(V, LD, 16 * ks, 32 * wave, lane);
            acc = mfma(vt, frag(Ph, LDP, j, 16 * ks + 8 * half), acc);
            acc = mfma(vt, frag(Pl, LDP, j, 16 * ks + 8 * half), acc);
        }
        res[jb] = pack_block(acc);
    }
    __syncthreads();  // every wave is done with Q
    _Pragma("unroll") for (int jb = 0; jb < 2; ++jb) store_packed(Q, LD, 32 * jb + n, 32 * wave, half, res[jb]);
    __syncthreads();
    store_tile_strided(o, Q, tok0, L, d.dv, D * vh, tid);
}
