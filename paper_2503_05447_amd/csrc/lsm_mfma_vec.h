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

// Chunk-local inclusive cumulative log-decay b [64][128] (fp32, row stride LDF) into LDS; tokens >= L
// carry g = 0.  Called by all 256 threads; ends with a barrier.
__device__ __forceinline__ void decay_tile(float* bt, const float* __restrict__ g, size_t tok0, int ts, int L, int tid) {
    const int cp = tid & 15, r0 = tid >> 4;
    _Pragma("unroll") for (int it = 0; it < 4; ++it) {
        const int row = r0 + 16 * it;
        // branch-free (rows beyond the ragged end read the last valid row and are zeroed): a branch
        // around a load makes the wave wait for every load in flight
        const float* src = g + (tok0 + size_t(min(row, L - 1)) * ts) * D + cp * 8;
        typedef float f32x4 __attribute__((ext_vector_type(4)));
        const f32x4 g0 = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(src));
        const f32x4 g1 = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(src + 4));
        const float keep = row < L ? 1.f : 0.f;
        *reinterpret_cast<float4*>(bt + row * LDF + cp * 8) = float4{g0.x * keep, g0.y * keep, g0.z * keep, g0.w * keep};
        *reinterpret_cast<float4*>(bt + row * LDF + cp * 8 + 4) = float4{g1.x * keep, g1.y * keep, g1.z * keep, g1.w * keep};
    }
    __syncthreads();
    // inclusive scan along tokens, one feature column per thread, two halves of 32 tokens
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
    __syncthreads();
}
// 8 consecutive floats of row `row` of the decay tile
__device__ __forceinline__ void decay_row8(const float* bt, int row, int col, float* out) {
    const float4 x0 = *reinterpret_cast<const float4*>(bt + row * LDF + col);
    const float4 x1 = *reinterpret_cast<const float4*>(bt + row * LDF + col + 4);
    out[0] = x0.x; out[1] = x0.y; out[2] = x0.z; out[3] = x0.w; out[4] = x1.x; out[5] = x1.y; out[6] = x1.z; out[7] = x1.w;
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
    const ChunkPos pos = chunk_pos(d, c, bh);
    const int L = pos.L;
    if (L <= 0) return;  // packed input: the grid is sized for an upper bound of the chunk count
    const size_t tok0 = pos.tok0, wtok0 = pos.wtok0;
    const int ts = pos.ts;
    const int n = lane & 31, half = lane >> 5;
    const int cp = tid & 15, r0 = tid >> 4;  // this thread's feature piece (8 features) and first row; rows r0 + 16 it

    // raw q, k pieces stay in registers for all levels
    u32x4 qr[4], kr[4];
    _Pragma("unroll") for (int it = 0; it < 4; ++it) {
        const int row = r0 + 16 * it;
        qr[it] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(q + (tok0 + size_t(min(row, L - 1)) * ts) * D + cp * 8));
        kr[it] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(k + (tok0 + size_t(min(row, L - 1)) * ts) * D + cp * 8));
    }
    decay_tile(bt, g, tok0, ts, L, tid);
    _Pragma("unroll") for (int it = 0; it < 4; ++it) {  // zero the ragged tail (after the loads have been issued)
        const uint32_t keep = r0 + 16 * it < L ? 0xffffffffu : 0u;
        qr[it] = u32x4{qr[it].x & keep, qr[it].y & keep, qr[it].z & keep, qr[it].w & keep};
        kr[it] = u32x4{kr[it].x & keep, kr[it].y & keep, kr[it].z & keep, kr[it].w & keep};
    }
    // diagonal scores q_t . k_t: exact products, summed over this thread's 8 features, then over the
    // 16 threads that share the row (consecutive lanes)
    _Pragma("unroll") for (int it = 0; it < 4; ++it) {
        float s = 0.f;
        _Pragma("unroll") for (int p = 0; p < 4; ++p)
            s += bf16_lo(qr[it][p]) * bf16_lo(kr[it][p]) + bf16_hi(qr[it][p]) * bf16_hi(kr[it][p]);
        _Pragma("unroll") for (int off = 8; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
        if (cp == 0) diag[r0 + 16 * it] = s;  // read after the barriers of the level loop
    }
    float bC[8];
    decay_row8(bt, 63, cp * 8, bC);
    auto brow = [&](int row, float* out) { decay_row8(bt, row, cp * 8, out); };
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
            *reinterpret_cast<u32x4*>(khat_hi + (wtok0 + row) * D + cp * 8) = hi;
            *reinterpret_cast<u32x4*>(khat_lo + (wtok0 + row) * D + cp * 8) = lo;
            weigh8(qr[it], wq, hi, &lo);
            *reinterpret_cast<u32x4*>(qhat_hi + (wtok0 + row) * D + cp * 8) = hi;
            *reinterpret_cast<u32x4*>(qhat_lo + (wtok0 + row) * D + cp * 8) = lo;
        }
    }
    if (tid < D) lamv[pos.slot * D + tid] = __expf(bt[63 * LDF + tid]);

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
        const size_t off = pos.slot * C * C + j * C + rbase;
        *reinterpret_cast<u32x4*>(p_hi + off) = hi[0];
        *reinterpret_cast<u32x4*>(p_hi + off + 8) = hi[1];
        *reinterpret_cast<u32x4*>(p_lo + off) = lo[0];
        *reinterpret_cast<u32x4*>(p_lo + off + 8) = lo[1];
    }
}

// 64 x 128 bf16 tile out of rows of `stride` elements starting at column `col0`; rows >= L zero
__device__ __forceinline__ void load_tile_strided(uint16_t* dst, const uint16_t* src, size_t tok0, int ts, int L, int stride,
                                                  int col0, int tid) {
    _Pragma("unroll") for (int it = 0; it < 4; ++it) {
        const int p = tid + kThreads * it, row = p >> 4, cp = p & 15;
        const u32x4 v = __builtin_nontemporal_load(
            reinterpret_cast<const u32x4*>(src + (tok0 + size_t(min(row, L - 1)) * ts) * stride + col0 + cp * 8));
        const uint32_t keep = row < L ? 0xffffffffu : 0u;
        *reinterpret_cast<u32x4*>(dst + row * LD + cp * 8) = u32x4{v.x & keep, v.y & keep, v.z & keep, v.w & keep};
    }
}
__device__ __forceinline__ void store_tile_strided(uint16_t* dst, const uint16_t* src, size_t tok0, int ts, int L, int stride,
                                                   int col0, int tid) {
    _Pragma("unroll") for (int it = 0; it < 4; ++it) {
        const int p = tid + kThreads * it, row = p >> 4, cp = p & 15;
        if (row < L)
            __builtin_nontemporal_store(*reinterpret_cast<const u32x4*>(src + row * LD + cp * 8),
                                        reinterpret_cast<u32x4*>(dst + (tok0 + size_t(row) * ts) * stride + col0 + cp * 8));
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
// DV = true computes with the same structure the value gradient
//   dv^T[v][r] = sum_i dS^T[v][i] khat_r[i] + sum_{j>=r} dO^T[v][j] P[j][r]
// (states = dS^T, qhat = khat, v = d_o; P is read through the LDS transpose read).
// LDS: qhat head (later the O stage) | qhat remainder | V slice | P head | P remainder
constexpr int kOutVecLds = 3 * C * LD * 2 + 2 * C * LDP * 2;

template <bool DV>
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
    const ChunkPos pos = chunk_pos(d, c, bh);
    const int L = pos.L;
    if (L <= 0) return;  // packed input: the grid is sized for an upper bound of the chunk count
    const size_t tok0 = pos.tok0, wtok0 = pos.wtok0;
    const int ts = pos.ts;
    const int n = lane & 31, half = lane >> 5;

    const uint16_t* St = states + (pos.slot * nvh + vh) * D * D;
    bf16x8 sfrag[8];
    _Pragma("unroll") for (int ks = 0; ks < 8; ++ks)
        sfrag[ks] = *reinterpret_cast<const bf16x8*>(St + state_frag_off(wave, ks, lane));

    load_tile(Q, qhat, wtok0, 1, L, tid);  // the library's own planes
    load_tile(Ql, qhat_lo, wtok0, 1, L, tid);
    load_tile_strided(V, v, tok0, ts, L, d.dv, D * vh, tid);
    const size_t poff = pos.slot * C * C;
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
        if (!DV) {
            _Pragma("unroll") for (int ks = 0; ks < 2 * (jb + 1); ++ks) {  // keys r >= 32 never reach queries j < 32
                const bf16x8 vt = frag_tr(V, LD, 16 * ks, 32 * wave, lane);
                acc = mfma(vt, frag(Ph, LDP, j, 16 * ks + 8 * half), acc);
                acc = mfma(vt, frag(Pl, LDP, j, 16 * ks + 8 * half), acc);
            }
        } else {
            _Pragma("unroll") for (int ks = 2 * jb; ks < 4; ++ks) {  // queries j < 32 never see keys r >= 32
                const bf16x8 vt = frag_tr(V, LD, 16 * ks, 32 * wave, lane);
                acc = mfma(vt, frag_tr(Ph, LDP, 16 * ks, 32 * jb, lane), acc);  // B[k = j][n = r] = P[j][r]
                acc = mfma(vt, frag_tr(Pl, LDP, 16 * ks, 32 * jb, lane), acc);
            }
        }
        res[jb] = pack_block(acc);
    }
    __syncthreads();  // every wave is done with Q
    _Pragma("unroll") for (int jb = 0; jb < 2; ++jb) store_packed(Q, LD, 32 * jb + n, 32 * wave, half, res[jb]);
    __syncthreads();
    store_tile_strided(o, Q, tok0, ts, L, d.dv, D * vh, tid);
}

// ---------------------------------------------------------------------------------------------
// dq, dk and the decay gradient of one chunk (grid: N x BH), vector decay kind.
//   dA[j][r] = d_o_j . v_r  (r <= j),   Z[u][t] = dA[max(u,t)][min(u,t)]  (symmetric, 64 x 64)
//   dq_j[i] = e^{b_j[i]} sum_v S[i][v] d_o_j[v]           + sum_{r<j} dA[j][r] k_r[i] e^{b_j[i]-b_r[i]} + dA[j][j] k_j[i]
//   dk_r[i] = e^{b_C[i]-b_r[i]} sum_v dS[i][v] v_r[v]     + sum_{j>r} dA[j][r] q_j[i] e^{b_j[i]-b_r[i]} + dA[r][r] q_r[i]
//   dg_t[i] = sum_{u>=t} (q_u[i] dq_u[i] - k_u[i] dk_u[i]) + sum_r k_r[i] dk_r^{inter}[i] + e^{b_C[i]} sum_v S[i][v] dS[i][v]
// The intra sums use the level tiles W_s of mk_vec_prep: at level s every token t is on one side, and
//   X_s[t][i] = sum_u Z_s[u][t] W_s[u][i]     (Z_s = Z restricted to the pairs of level s)
// times the token's own level weight is its contribution to dq_t (t on the query side) or dk_t (key
// side).  Wave w owns features [32w, 32w+32) of dq^T, dk^T (D layout: lane = token, registers =
// features).  Z is built once (wave 0, 1: the diagonal 32-blocks, wave 2, 3: the off-diagonal ones),
// summed over the 128-wide value slices, and kept in LDS as bf16 head + remainder.
// LDS: b | Q | K | T0 (V slice, then W head, then dq stage) | T1 (d_o slice, W remainder, dk stage)
//      | Z head | Z remainder | diagonal of dA | <S,dS> per feature
constexpr int kGradVecLds = C * LDF * 4 + 4 * C * LD * 2 + 2 * C * LDP * 2 + C * 4 + D * 4;

__global__ __launch_bounds__(kThreads, 1) void mk_grad_vec(Dims d, const uint16_t* __restrict__ q,
                                                           const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
                                                           const uint16_t* __restrict__ d_o, const float* __restrict__ g,
                                                           const uint16_t* __restrict__ states,
                                                           const uint16_t* __restrict__ states_rem,
                                                           const uint16_t* __restrict__ dstates,
                                                           const uint16_t* __restrict__ dstates_rem,
                                                           uint16_t* __restrict__ dq, uint16_t* __restrict__ dk,
                                                           float* __restrict__ dg) {
    extern __shared__ __align__(16) unsigned char smem[];
    float* bt = reinterpret_cast<float*>(smem);
    uint16_t* Qr = reinterpret_cast<uint16_t*>(bt + C * LDF);
    uint16_t* Kr = Qr + C * LD;
    uint16_t* T0 = Kr + C * LD;
    uint16_t* T1 = T0 + C * LD;
    uint16_t* Zh = T1 + C * LD;
    uint16_t* Zl = Zh + C * LDP;
    float* zd = reinterpret_cast<float*>(Zl + C * LDP);  // [64]
    float* zl = zd + C;                                  // [128]

    const int c = blockIdx.x, bh = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const ChunkPos pos = chunk_pos(d, c, bh);
    const int L = pos.L;
    if (L <= 0) return;  // packed input: the grid is sized for an upper bound of the chunk count
    const size_t tok0 = pos.tok0, wtok0 = pos.wtok0;
    const int ts = pos.ts;
    const int n = lane & 31, half = lane >> 5;
    const int nvh = d.dv / D;
    const bool want_dg = dg != nullptr;  // then states_rem and dstates_rem are present

    // Global loads are issued as early and as many at a time as the registers allow: with one
    // workgroup per CU nothing else hides their latency.  Per value slice: the V and d_o tiles (via
    // registers into LDS) and this wave's rows of S, dS and their remainder planes (MFMA A operands).
    struct SliceRegs {
        u32x4 tv[4], to[4];
        bf16x8 s[8], ds[8];
        u32x2 sr[8], dsr[8];  // remainder planes: 8-bit floats, still scaled by 2^8
    };
    auto issue = [&](int vh, SliceRegs& r) {
        _Pragma("unroll") for (int it = 0; it < 4; ++it) {
            const int p = tid + kThreads * it, row = p >> 4, cpp = p & 15;
            const size_t off = (tok0 + size_t(min(row, L - 1)) * ts) * d.dv + D * vh + cpp * 8;
            const uint32_t keep = row < L ? 0xffffffffu : 0u;
            u32x4 a = *reinterpret_cast<const u32x4*>(v + off), b = *reinterpret_cast<const u32x4*>(d_o + off);
            r.tv[it] = u32x4{a.x & keep, a.y & keep, a.z & keep, a.w & keep};
            r.to[it] = u32x4{b.x & keep, b.y & keep, b.z & keep, b.w & keep};
        }
        const size_t sbase = (pos.slot * nvh + vh) * D * D;
        _Pragma("unroll") for (int ks = 0; ks < 8; ++ks) {
            const size_t soff = sbase + state_frag_off(wave, ks, lane);
            r.s[ks] = *reinterpret_cast<const bf16x8*>(states + soff);
            r.ds[ks] = *reinterpret_cast<const bf16x8*>(dstates + soff);
            if (want_dg) {
                r.sr[ks] = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(reinterpret_cast<const uint8_t*>(states_rem) + soff));
                r.dsr[ks] = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(reinterpret_cast<const uint8_t*>(dstates_rem) + soff));
            }
        }
    };
    auto commit = [&](const SliceRegs& r) {
        _Pragma("unroll") for (int it = 0; it < 4; ++it) {
            const int p = tid + kThreads * it, row = p >> 4, cpp = p & 15;
            *reinterpret_cast<u32x4*>(T0 + row * LD + cpp * 8) = r.tv[it];
            *reinterpret_cast<u32x4*>(T1 + row * LD + cpp * 8) = r.to[it];
        }
    };
    SliceRegs sr0;
    load_tile(Qr, q, tok0, ts, L, tid);
    load_tile(Kr, k, tok0, ts, L, tid);
    issue(0, sr0);
    decay_tile(bt, g, tok0, ts, L, tid);

    // ---- inter parts and Z, slice by slice of the value dimension
    // aqr, akr: contributions of the remainder planes of S and dS; they enter the decay gradient only, so
    // that dq and dk do not depend on whether it is asked for
    f32x16 aq[2] = {{0}, {0}}, aqr[2] = {{0}, {0}}, ak[2] = {{0}, {0}}, akr[2] = {{0}, {0}};
    f32x16 z0 = {0}, z1 = {0};
    float zi = 0.f;
    for (int vh = 0; vh < nvh; ++vh) {
        if (vh > 0) {
            __syncthreads();  // the previous slice is consumed
            issue(vh, sr0);
        }
        commit(sr0);
        __syncthreads();
        _Pragma("unroll") for (int nb = 0; nb < 2; ++nb)
            _Pragma("unroll") for (int ks = 0; ks < 8; ++ks) {
                const bf16x8 dof = frag(T1, LD, 32 * nb + n, 16 * ks + 8 * half), vf = frag(T0, LD, 32 * nb + n, 16 * ks + 8 * half);
                aq[nb] = mfma(sr0.s[ks], dof, aq[nb]);
                ak[nb] = mfma(sr0.ds[ks], vf, ak[nb]);
                if (want_dg) {
                    aqr[nb] = mfma(rem8_to_bf16(sr0.sr[ks]), dof, aqr[nb]);
                    akr[nb] = mfma(rem8_to_bf16(sr0.dsr[ks]), vf, akr[nb]);
                }
            }
        if (want_dg) {  // <S, dS> over this lane's share of row i = 32 wave + n
            _Pragma("unroll") for (int ks = 0; ks < 8; ++ks) {
                const u32x4 a = __builtin_bit_cast(u32x4, sr0.s[ks]), ar = __builtin_bit_cast(u32x4, rem8_to_bf16(sr0.sr[ks]));
                const u32x4 b = __builtin_bit_cast(u32x4, sr0.ds[ks]), br = __builtin_bit_cast(u32x4, rem8_to_bf16(sr0.dsr[ks]));
                _Pragma("unroll") for (int p = 0; p < 4; ++p)
                    zi += (bf16_lo(a[p]) + kRem8Unscale * bf16_lo(ar[p])) * (bf16_lo(b[p]) + kRem8Unscale * bf16_lo(br[p])) +
                          (bf16_hi(a[p]) + kRem8Unscale * bf16_hi(ar[p])) * (bf16_hi(b[p]) + kRem8Unscale * bf16_hi(br[p]));
            }
        }
        {   // this wave's block of Z: rows of V and d_o as operands
            const int rowv = wave == 1 ? 32 + n : n;               // V row: wave 0, 2, 3: 0.., wave 1: 32..
            const int rowo = wave == 0 ? n : 32 + n;               // d_o row: wave 0: 0.., else 32..
            _Pragma("unroll") for (int ks = 0; ks < 8; ++ks) {
                const bf16x8 fv = frag(T0, LD, rowv, 16 * ks + 8 * half), fo = frag(T1, LD, rowo, 16 * ks + 8 * half);
                if (wave == 3) z0 = mfma(fo, fv, z0);              // D[m][n] = d_o_{32+m} . v_n
                else z0 = mfma(fv, fo, z0);                        // D[m][n] = v_m . d_o_n
                if (wave < 2) z1 = mfma(fo, fv, z1);               // D[m][n] = d_o_m . v_n
            }
        }
    }
    {   // Z[u][t] -> LDS rows t, head and remainder; diagonal of dA
        const int ub = (wave == 1 || wave == 3) ? 1 : 0, tb = (wave == 1 || wave == 2) ? 1 : 0;
        if (wave < 2) {
            _Pragma("unroll") for (int x = 0; x < 16; ++x) {
                const int m = 8 * (x >> 2) + 4 * half + (x & 3);
                if (m == n) zd[32 * wave + n] = z0[x];
                z0[x] = m <= n ? z0[x] : z1[x];
            }
        }
        store_block_t_split(Zh, Zl, LDP, 32 * tb + n, 32 * ub, half, z0);
    }
    // weights of the inter parts; the part of dg that needs dk^{inter}
    f32x16 xk = {0};
    _Pragma("unroll") for (int nb = 0; nb < 2; ++nb) {
        const int t = 32 * nb + n;
        _Pragma("unroll") for (int gq = 0; gq < 4; ++gq) {
            const int col = 32 * wave + 8 * gq + 4 * half;
            const float4 b4 = *reinterpret_cast<const float4*>(bt + t * LDF + col);
            const float4 c4 = *reinterpret_cast<const float4*>(bt + 63 * LDF + col);
            const float bb[4] = {b4.x, b4.y, b4.z, b4.w}, cc[4] = {c4.x, c4.y, c4.z, c4.w};
            const u32x2 kk = *reinterpret_cast<const u32x2*>(Kr + t * LD + col);
            const float kf[4] = {bf16_lo(kk.x), bf16_hi(kk.x), bf16_lo(kk.y), bf16_hi(kk.y)};
            _Pragma("unroll") for (int jj = 0; jj < 4; ++jj) {
                const int x = 4 * gq + jj;
                const float wq = __expf(bb[jj]), wk = __expf(cc[jj] - bb[jj]);
                aq[nb][x] *= wq;
                aqr[nb][x] *= wq * kRem8Unscale;
                ak[nb][x] *= wk;
                akr[nb][x] *= wk * kRem8Unscale;
                xk[x] += kf[jj] * (ak[nb][x] + akr[nb][x]);
            }
        }
    }
    if (want_dg) {
        zi += __shfl_xor(zi, 32, 64);
        if (half == 0) zl[32 * wave + n] = zi;
    }

    // ---- levels
    const int cp = tid & 15, r0 = tid >> 4;
    _Pragma("unroll") for (int lv = 0; lv < 6; ++lv) {
        const int ls = 5 - lv;
        __syncthreads();  // lv = 0: Z complete, V / d_o slices consumed; else: the previous level's tiles are read
        _Pragma("unroll") for (int it = 0; it < 4; ++it) {
            const int row = r0 + 16 * it;
            bool qside;
            const int ref = level_ref(row, ls, qside);
            float b[8], br[8], w[8];
            decay_row8(bt, row, cp * 8, b);
            decay_row8(bt, ref, cp * 8, br);
            _Pragma("unroll") for (int e = 0; e < 8; ++e) w[e] = __expf(qside ? b[e] - br[e] : br[e] - b[e]);
            const u32x4 raw = *reinterpret_cast<const u32x4*>((qside ? Qr : Kr) + row * LD + cp * 8);
            u32x4 hi, lo;
            weigh8(raw, w, hi, &lo);
            *reinterpret_cast<u32x4*>(T0 + row * LD + cp * 8) = hi;
            *reinterpret_cast<u32x4*>(T1 + row * LD + cp * 8) = lo;
        }
        __syncthreads();
        _Pragma("unroll") for (int nb = 0; nb < 2; ++nb) {
            const int t = 32 * nb + n;
            const int ub = ls == 5 ? 1 - nb : nb;  // the partners of level 32 sit in the other 32-block
            f32x16 X = {0};
            _Pragma("unroll") for (int s2 = 0; s2 < 2; ++s2) {
                const int u0 = 32 * ub + 16 * s2;
                const int xr = (u0 + 8 * half) ^ t;
                u32x4 mask;
                _Pragma("unroll") for (int p = 0; p < 4; ++p)
                    mask[p] = ((((xr ^ (2 * p)) >> ls) == 1) ? 0xffffu : 0u) | ((((xr ^ (2 * p + 1)) >> ls) == 1) ? 0xffff0000u : 0u);
                u32x4 zh = *reinterpret_cast<const u32x4*>(Zh + t * LDP + u0 + 8 * half);
                u32x4 zlo = *reinterpret_cast<const u32x4*>(Zl + t * LDP + u0 + 8 * half);
                _Pragma("unroll") for (int p = 0; p < 4; ++p) {
                    zh[p] &= mask[p];
                    zlo[p] &= mask[p];
                }
                const bf16x8 bzh = __builtin_bit_cast(bf16x8, zh), bzl = __builtin_bit_cast(bf16x8, zlo);
                const bf16x8 ah = frag_tr(T0, LD, u0, 32 * wave, lane), al = frag_tr(T1, LD, u0, 32 * wave, lane);
                X = mfma(ah, bzh, X);
                X = mfma(ah, bzl, X);
                X = mfma(al, bzh, X);
            }
            bool qside;
            const int ref = level_ref(t, ls, qside);
            _Pragma("unroll") for (int gq = 0; gq < 4; ++gq) {
                const int col = 32 * wave + 8 * gq + 4 * half;
                const float4 b4 = *reinterpret_cast<const float4*>(bt + t * LDF + col);
                const float4 r4 = *reinterpret_cast<const float4*>(bt + ref * LDF + col);
                const float bb[4] = {b4.x, b4.y, b4.z, b4.w}, rr[4] = {r4.x, r4.y, r4.z, r4.w};
                _Pragma("unroll") for (int jj = 0; jj < 4; ++jj) {
                    const int x = 4 * gq + jj;
                    const float val = X[x] * __expf(qside ? bb[jj] - rr[jj] : rr[jj] - bb[jj]);
                    aq[nb][x] += qside ? val : 0.f;
                    ak[nb][x] += qside ? 0.f : val;
                }
            }
        }
    }
    // ---- diagonal pairs, then the decay gradient from the unrounded accumulators
    f32x16 wd[2];
    _Pragma("unroll") for (int nb = 0; nb < 2; ++nb) {
        const int t = 32 * nb + n;
        const float dd = zd[t];
        _Pragma("unroll") for (int gq = 0; gq < 4; ++gq) {
            const int col = 32 * wave + 8 * gq + 4 * half;
            const u32x2 qq = *reinterpret_cast<const u32x2*>(Qr + t * LD + col);
            const u32x2 kk = *reinterpret_cast<const u32x2*>(Kr + t * LD + col);
            const float qf[4] = {bf16_lo(qq.x), bf16_hi(qq.x), bf16_lo(qq.y), bf16_hi(qq.y)};
            const float kf[4] = {bf16_lo(kk.x), bf16_hi(kk.x), bf16_lo(kk.y), bf16_hi(kk.y)};
            _Pragma("unroll") for (int jj = 0; jj < 4; ++jj) {
                const int x = 4 * gq + jj;
                aq[nb][x] += dd * kf[jj];
                ak[nb][x] += dd * qf[jj];
                wd[nb][x] = qf[jj] * (aq[nb][x] + aqr[nb][x]) - kf[jj] * (ak[nb][x] + akr[nb][x]);
            }
        }
    }
    __syncthreads();  // every wave is done with the level tiles and with b as weights
    _Pragma("unroll") for (int nb = 0; nb < 2; ++nb) {
        store_packed(T0, LD, 32 * nb + n, 32 * wave, half, pack_block(aq[nb]));
        store_packed(T1, LD, 32 * nb + n, 32 * wave, half, pack_block(ak[nb]));
    }
    if (want_dg) {
        // per feature (register): inclusive suffix sum over the tokens (lanes of one half), block 1 first
        _Pragma("unroll") for (int nb = 1; nb >= 0; --nb) {
            _Pragma("unroll") for (int off = 1; off < 32; off <<= 1) {
                _Pragma("unroll") for (int x = 0; x < 16; ++x) {
                    const float y = __shfl_down(wd[nb][x], off, 32);
                    wd[nb][x] += (n + off < 32) ? y : 0.f;
                }
            }
            if (nb == 1) {
                _Pragma("unroll") for (int x = 0; x < 16; ++x) {
                    const float total = __shfl(wd[1][x], 0, 32);  // all lanes take part in the exchange
                    wd[0][x] += (n == 31) ? total : 0.f;
                }
            }
        }
        _Pragma("unroll") for (int off = 1; off < 32; off <<= 1) {
            _Pragma("unroll") for (int x = 0; x < 16; ++x) xk[x] += __shfl_xor(xk[x], off, 32);
        }
        _Pragma("unroll") for (int gq = 0; gq < 4; ++gq) {
            const int col = 32 * wave + 8 * gq + 4 * half;
            const float4 c4 = *reinterpret_cast<const float4*>(bt + 63 * LDF + col);
            const float4 z4 = *reinterpret_cast<const float4*>(zl + col);
            const float cc[4] = {c4.x, c4.y, c4.z, c4.w}, zz[4] = {z4.x, z4.y, z4.z, z4.w};
            _Pragma("unroll") for (int jj = 0; jj < 4; ++jj) xk[4 * gq + jj] += __expf(cc[jj]) * zz[jj];
        }
    }
    __syncthreads();  // stages complete; b no longer needed
    store_tile(dq, T0, tok0, ts, L, tid);
    store_tile(dk, T1, tok0, ts, L, tid);
    if (want_dg) {
        _Pragma("unroll") for (int nb = 0; nb < 2; ++nb)
            _Pragma("unroll") for (int gq = 0; gq < 4; ++gq)
                *reinterpret_cast<float4*>(bt + (32 * nb + n) * LDF + 32 * wave + 8 * gq + 4 * half) =
                    float4{wd[nb][4 * gq] + xk[4 * gq], wd[nb][4 * gq + 1] + xk[4 * gq + 1],
                           wd[nb][4 * gq + 2] + xk[4 * gq + 2], wd[nb][4 * gq + 3] + xk[4 * gq + 3]};
        __syncthreads();
        _Pragma("unroll") for (int it = 0; it < 8; ++it) {
            const int p = tid + kThreads * it, row = p >> 5, c4 = p & 31;
            if (row < L)
                *reinterpret_cast<float4*>(dg + (tok0 + size_t(row) * ts) * D + 4 * c4) = *reinterpret_cast<const float4*>(bt + row * LDF + 4 * c4);
        }
    }
}
