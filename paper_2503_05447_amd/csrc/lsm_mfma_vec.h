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

    const int c = blockIdx.x, bh = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
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
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
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
// side).  Eight waves: wave (w, nb) owns features [32w, 32w+32) of dq^T, dk^T for the tokens
// [32nb, 32nb+32) (D layout: lane = token, registers = features), so that two waves share a SIMD
// and the long per-element weight arithmetic of one overlaps the waits of the other.  Z is built
// once (waves 0..3: one 32 x 32 block each), summed over the 128-wide value slices, and kept in LDS
// as bf16 head + remainder.
// LDS: b | Q | K | T0 (V slice, then W head, then dq stage) | T1 (d_o slice, W remainder, dk stage)
//      | Z head | Z remainder | diagonal of dA | <S,dS> per feature | exchange between the two token blocks
//      | second level-tile buffer (head, remainder)        -- 155 KiB in all
constexpr int kGradVecThreads = 512;
constexpr int kGradVecLds = C * LDF * 4 + 6 * C * LD * 2 + 2 * C * LDP * 2 + C * 4 + D * 4 + 3 * 4 * 32 * 4;

__global__ __launch_bounds__(kGradVecThreads, 1) void mk_grad_vec(Dims d, const uint16_t* __restrict__ q,
                                                                  const uint16_t* __restrict__ k,
                                                                  const uint16_t* __restrict__ v,
                                                                  const uint16_t* __restrict__ d_o,
                                                                  const float* __restrict__ g,
                                                                  const uint16_t* __restrict__ states,
                                                                  const uint16_t* __restrict__ states_rem,
                                                                  const uint16_t* __restrict__ dstates,
                                                                  const uint16_t* __restrict__ dstates_rem,
                                                                  uint16_t* __restrict__ dq, uint16_t* __restrict__ dk,
                                                                  float* __restrict__ dg) {
    constexpr int NT = kGradVecThreads;
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
    float* xch = zl + D;                                 // [3][4][32]: block-1 totals of the running sum, tail sums of both blocks
    uint16_t* W1 = reinterpret_cast<uint16_t*>(xch + 3 * 4 * 32);  // second level-tile buffer: head | remainder

    const int c = blockIdx.x, bh = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int wave = wv & 3, nb = wv >> 2;  // feature block, token block
    const ChunkPos pos = chunk_pos(d, c, bh);
    const int L = pos.L;
    if (L <= 0) return;  // packed input: the grid is sized for an upper bound of the chunk count
    const size_t tok0 = pos.tok0;
    const int ts = pos.ts;
    const int n = lane & 31, half = lane >> 5;
    const int t = 32 * nb + n;  // this lane's token
    const int nvh = d.dv / D;
    const bool want_dg = dg != nullptr;  // then states_rem and dstates_rem are present

    // 64 x 128 tiles move as 1024 16-byte pieces, two per thread
    auto tile_rows = [&](int it, int& row, int& cpp) { const int p = tid + NT * it; row = p >> 4; cpp = p & 15; };
    struct SliceRegs {
        u32x4 tv[2], to[2];
        bf16x8 s[8], ds[8];
        u32x2 sr[8], dsr[8];  // remainder planes: 8-bit floats, still scaled by 2^8
    };
    auto issue = [&](int vh, SliceRegs& r) {
        _Pragma("unroll") for (int it = 0; it < 2; ++it) {
            int row, cpp;
            tile_rows(it, row, cpp);
            const size_t off = (tok0 + size_t(min(row, L - 1)) * ts) * d.dv + D * vh + cpp * 8;
            r.tv[it] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(v + off));
            r.to[it] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(d_o + off));
        }
        // this wave's rows of S, dS (both token blocks read the same rows) and their 8-bit remainder planes
        const size_t sbase = (pos.slot * nvh + vh) * D * D;
        _Pragma("unroll") for (int ks = 0; ks < 8; ++ks) {
            const size_t soff = sbase + state_frag_off(wave, ks, lane);
            r.s[ks] = *reinterpret_cast<const bf16x8*>(states + soff);
            r.ds[ks] = *reinterpret_cast<const bf16x8*>(dstates + soff);
            if (want_dg) {
                r.sr[ks] = *reinterpret_cast<const u32x2*>(reinterpret_cast<const uint8_t*>(states_rem) + soff);
                r.dsr[ks] = *reinterpret_cast<const u32x2*>(reinterpret_cast<const uint8_t*>(dstates_rem) + soff);
            }
        }
    };
    auto commit = [&](const SliceRegs& r) {
        _Pragma("unroll") for (int it = 0; it < 2; ++it) {
            int row, cpp;
            tile_rows(it, row, cpp);
            const uint32_t keep = row < L ? 0xffffffffu : 0u;
            *reinterpret_cast<u32x4*>(T0 + row * LD + cpp * 8) = u32x4{r.tv[it].x & keep, r.tv[it].y & keep, r.tv[it].z & keep, r.tv[it].w & keep};
            *reinterpret_cast<u32x4*>(T1 + row * LD + cpp * 8) = u32x4{r.to[it].x & keep, r.to[it].y & keep, r.to[it].z & keep, r.to[it].w & keep};
        }
    };
    // ---- q, k, g and the first value slice: every load issued before the first wait
    SliceRegs sr0;
    {
        u32x4 tq[2], tk[2];
        typedef float f32x4 __attribute__((ext_vector_type(4)));
        f32x4 tg[2][2];
        _Pragma("unroll") for (int it = 0; it < 2; ++it) {
            int row, cpp;
            tile_rows(it, row, cpp);
            const size_t roff = (tok0 + size_t(min(row, L - 1)) * ts) * D + cpp * 8;
            tq[it] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(q + roff));
            tk[it] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(k + roff));
            tg[it][0] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(g + roff));
            tg[it][1] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(g + roff + 4));
        }
        issue(0, sr0);
        _Pragma("unroll") for (int it = 0; it < 2; ++it) {
            int row, cpp;
            tile_rows(it, row, cpp);
            const uint32_t keep = row < L ? 0xffffffffu : 0u;
            const float kf = row < L ? 1.f : 0.f;
            *reinterpret_cast<u32x4*>(Qr + row * LD + cpp * 8) = u32x4{tq[it].x & keep, tq[it].y & keep, tq[it].z & keep, tq[it].w & keep};
            *reinterpret_cast<u32x4*>(Kr + row * LD + cpp * 8) = u32x4{tk[it].x & keep, tk[it].y & keep, tk[it].z & keep, tk[it].w & keep};
            *reinterpret_cast<float4*>(bt + row * LDF + cpp * 8) = float4{tg[it][0].x * kf, tg[it][0].y * kf, tg[it][0].z * kf, tg[it][0].w * kf};
            *reinterpret_cast<float4*>(bt + row * LDF + cpp * 8 + 4) = float4{tg[it][1].x * kf, tg[it][1].y * kf, tg[it][1].z * kf, tg[it][1].w * kf};
        }
    }
    __syncthreads();
    {   // inclusive scan of g along tokens: one feature column per thread, four quarters of 16 tokens
        const int i = tid & 127, hq = tid >> 7;
        float run = 0.f;
        for (int r = 16 * hq; r < 16 * hq + 16; ++r) {
            run += bt[r * LDF + i];
            bt[r * LDF + i] = run;
        }
        __syncthreads();
        float base = 0.f;
        for (int qq = 0; qq < hq; ++qq) base += bt[(16 * qq + 15) * LDF + i];
        __syncthreads();
        if (hq > 0)
            for (int r = 16 * hq; r < 16 * hq + 16; ++r) bt[r * LDF + i] += base;
    }
    __syncthreads();

    // ---- inter parts and Z, slice by slice of the value dimension
    // aqr, akr: contributions of the remainder planes of S and dS; they enter the decay gradient only, so
    // that dq and dk do not depend on whether it is asked for
    f32x16 aq = {0}, aqr = {0}, ak = {0}, akr = {0};
    f32x16 z0 = {0}, z1 = {0};
    float zi = 0.f;
    for (int vh = 0; vh < nvh; ++vh) {
        if (vh > 0) {
            __syncthreads();  // the previous slice is consumed
            issue(vh, sr0);
        }
        commit(sr0);
        __syncthreads();
        _Pragma("unroll") for (int ks = 0; ks < 8; ++ks) {
            const bf16x8 sf = sr0.s[ks], dsf = sr0.ds[ks];
            const bf16x8 dof = frag(T1, LD, t, 16 * ks + 8 * half), vf = frag(T0, LD, t, 16 * ks + 8 * half);
            aq = mfma(sf, dof, aq);
            ak = mfma(dsf, vf, ak);
            if (want_dg) {
                const bf16x8 srf = rem8_to_bf16(sr0.sr[ks]), dsrf = rem8_to_bf16(sr0.dsr[ks]);
                aqr = mfma(srf, dof, aqr);
                akr = mfma(dsrf, vf, akr);
                if (nb == 0) {  // <S, dS> over this lane's share of row i = 32 wave + n
                    const u32x4 a = __builtin_bit_cast(u32x4, sf), ar = __builtin_bit_cast(u32x4, srf);
                    const u32x4 b = __builtin_bit_cast(u32x4, dsf), br = __builtin_bit_cast(u32x4, dsrf);
                    _Pragma("unroll") for (int p = 0; p < 4; ++p)
                        zi += (bf16_lo(a[p]) + kRem8Unscale * bf16_lo(ar[p])) * (bf16_lo(b[p]) + kRem8Unscale * bf16_lo(br[p])) +
                              (bf16_hi(a[p]) + kRem8Unscale * bf16_hi(ar[p])) * (bf16_hi(b[p]) + kRem8Unscale * bf16_hi(br[p]));
                }
            }
        }
        if (wv < 4) {  // this wave's block of Z: rows of V and d_o as operands
            const int rowv = wv == 1 ? 32 + n : n;               // V row: wave 0, 2, 3: 0.., wave 1: 32..
            const int rowo = wv == 0 ? n : 32 + n;               // d_o row: wave 0: 0.., else 32..
            _Pragma("unroll") for (int ks = 0; ks < 8; ++ks) {
                const bf16x8 fv = frag(T0, LD, rowv, 16 * ks + 8 * half), fo = frag(T1, LD, rowo, 16 * ks + 8 * half);
                if (wv == 3) z0 = mfma(fo, fv, z0);              // D[m][n] = d_o_{32+m} . v_n
                else z0 = mfma(fv, fo, z0);                      // D[m][n] = v_m . d_o_n
                if (wv < 2) z1 = mfma(fo, fv, z1);               // D[m][n] = d_o_m . v_n
            }
        }
    }
    if (wv < 4) {  // Z[u][t] -> LDS rows t, head and remainder; diagonal of dA
        const int ub = (wv == 1 || wv == 3) ? 1 : 0, tb = (wv == 1 || wv == 2) ? 1 : 0;
        if (wv < 2) {
            _Pragma("unroll") for (int x = 0; x < 16; ++x) {
                const int m = 8 * (x >> 2) + 4 * half + (x & 3);
                if (m == n) zd[32 * wv + n] = z0[x];
                z0[x] = m <= n ? z0[x] : z1[x];
            }
        }
        store_block_t_split(Zh, Zl, LDP, 32 * tb + n, 32 * ub, half, z0);
    }
    // weights of the inter parts; the part of dg that needs dk^{inter}
    f32x16 xk = {0};
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
            aq[x] *= wq;
            aqr[x] *= wq * kRem8Unscale;
            ak[x] *= wk;
            akr[x] *= wk * kRem8Unscale;
            xk[x] = kf[jj] * (ak[x] + akr[x]);
        }
    }
    if (want_dg && nb == 0) {
        zi += __shfl_xor(zi, 32, 64);
        if (half == 0) zl[32 * wave + n] = zi;
    }

    // ---- levels.  The level tiles are double-buffered, and the two waves of a SIMD (same features,
    // token blocks 0 and 1) take the two halves of an iteration in opposite order: while one builds
    // the tile of the next level (exponentials on the vector ALU) the other contracts the current one
    // (LDS reads, MFMA), instead of both queueing for the same unit.
    const int cp = tid & 15, r0 = tid >> 4;  // W rows r0 and r0 + 32, features 8 cp .. + 7
    auto Wh = [&](int lv) { return (lv & 1) ? W1 : T0; };
    auto Wl = [&](int lv) { return (lv & 1) ? W1 + C * LD : T1; };
    auto build = [&](int lv) {
        const int ls = 5 - lv;
        uint16_t *wh = Wh(lv), *wl = Wl(lv);
        _Pragma("unroll") for (int it = 0; it < 2; ++it) {
            const int row = r0 + 32 * it;
            bool qside;
            const int ref = level_ref(row, ls, qside);
            float b[8], br[8], w[8];
            decay_row8(bt, row, cp * 8, b);
            decay_row8(bt, ref, cp * 8, br);
            _Pragma("unroll") for (int e = 0; e < 8; ++e) w[e] = __expf(qside ? b[e] - br[e] : br[e] - b[e]);
            const u32x4 raw = *reinterpret_cast<const u32x4*>((qside ? Qr : Kr) + row * LD + cp * 8);
            u32x4 hi, lo;
            weigh8(raw, w, hi, &lo);
            *reinterpret_cast<u32x4*>(wh + row * LD + cp * 8) = hi;
            *reinterpret_cast<u32x4*>(wl + row * LD + cp * 8) = lo;
        }
    };
    auto contract = [&](int lv) {
        const int ls = 5 - lv;
        const uint16_t *wh = Wh(lv), *wl = Wl(lv);
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
            const bf16x8 ah = frag_tr(wh, LD, u0, 32 * wave, lane), al = frag_tr(wl, LD, u0, 32 * wave, lane);
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
                aq[x] += qside ? val : 0.f;
                ak[x] += qside ? 0.f : val;
            }
        }
    };
    __syncthreads();  // Z complete, V / d_o slices consumed
    build(0);
    __syncthreads();
    _Pragma("unroll") for (int lv = 0; lv < 6; ++lv) {
        if (nb == 0) {
            if (lv < 5) build(lv + 1);
            contract(lv);
        } else {
            contract(lv);
            if (lv < 5) build(lv + 1);
        }
        __syncthreads();  // the next tile is complete, this one is free again
    }
    // ---- diagonal pairs, then the decay gradient from the unrounded accumulators
    f32x16 wd;
    {
        const float dd = zd[t];
        _Pragma("unroll") for (int gq = 0; gq < 4; ++gq) {
            const int col = 32 * wave + 8 * gq + 4 * half;
            const u32x2 qq = *reinterpret_cast<const u32x2*>(Qr + t * LD + col);
            const u32x2 kk = *reinterpret_cast<const u32x2*>(Kr + t * LD + col);
            const float qf[4] = {bf16_lo(qq.x), bf16_hi(qq.x), bf16_lo(qq.y), bf16_hi(qq.y)};
            const float kf[4] = {bf16_lo(kk.x), bf16_hi(kk.x), bf16_lo(kk.y), bf16_hi(kk.y)};
            _Pragma("unroll") for (int jj = 0; jj < 4; ++jj) {
                const int x = 4 * gq + jj;
                aq[x] += dd * kf[jj];
                ak[x] += dd * qf[jj];
                wd[x] = qf[jj] * (aq[x] + aqr[x]) - kf[jj] * (ak[x] + akr[x]);
            }
        }
    }
    // (the barrier that ends the level loop: every wave is done with the level tiles)
    store_packed(T0, LD, t, 32 * wave, half, pack_block(aq));
    store_packed(T1, LD, t, 32 * wave, half, pack_block(ak));
    if (want_dg) {
        // per feature (register): inclusive suffix sum over this wave's 32 tokens (lanes of one half), the
        // sum of this wave's tail terms; both go to the other token block through LDS
        _Pragma("unroll") for (int off = 1; off < 32; off <<= 1) {
            _Pragma("unroll") for (int x = 0; x < 16; ++x) {
                const float y = __shfl_down(wd[x], off, 32);
                wd[x] += (n + off < 32) ? y : 0.f;
            }
        }
        _Pragma("unroll") for (int off = 1; off < 32; off <<= 1) {
            _Pragma("unroll") for (int x = 0; x < 16; ++x) xk[x] += __shfl_xor(xk[x], off, 32);
        }
        if (n == 0) {
            _Pragma("unroll") for (int x = 0; x < 16; ++x) {
                const int f = 8 * (x >> 2) + 4 * half + (x & 3);
                if (nb == 1) xch[(0 * 4 + wave) * 32 + f] = wd[x];   // total of token block 1
                xch[((1 + nb) * 4 + wave) * 32 + f] = xk[x];           // tail sum of this block
            }
        }
    }
    __syncthreads();  // stages and exchange complete; b no longer needed as weights
    {
        int row, cpp;
        _Pragma("unroll") for (int it = 0; it < 2; ++it) {
            tile_rows(it, row, cpp);
            if (row < L) {
                __builtin_nontemporal_store(*reinterpret_cast<const u32x4*>(T0 + row * LD + cpp * 8),
                                            reinterpret_cast<u32x4*>(dq + (tok0 + size_t(row) * ts) * D + cpp * 8));
                __builtin_nontemporal_store(*reinterpret_cast<const u32x4*>(T1 + row * LD + cpp * 8),
                                            reinterpret_cast<u32x4*>(dk + (tok0 + size_t(row) * ts) * D + cpp * 8));
            }
        }
    }
    if (want_dg) {
        float add[16];
        _Pragma("unroll") for (int gq = 0; gq < 4; ++gq) {
            const int col = 32 * wave + 8 * gq + 4 * half;
            const float4 c4 = *reinterpret_cast<const float4*>(bt + 63 * LDF + col);
            const float4 z4 = *reinterpret_cast<const float4*>(zl + col);
            const float cc[4] = {c4.x, c4.y, c4.z, c4.w}, zz[4] = {z4.x, z4.y, z4.z, z4.w};
            _Pragma("unroll") for (int jj = 0; jj < 4; ++jj) {
                const int x = 4 * gq + jj, f = 8 * gq + 4 * half + jj;
                // tail over all 64 tokens (block 0 first), the state term, and for block 0 the running sum of block 1
                add[x] = (xch[(1 * 4 + wave) * 32 + f] + xch[(2 * 4 + wave) * 32 + f]) + __expf(cc[jj]) * zz[jj] +
                         (nb == 0 ? xch[(0 * 4 + wave) * 32 + f] : 0.f);
            }
        }
        __syncthreads();  // every wave has read b and the exchange area: b becomes the dg stage
        _Pragma("unroll") for (int gq = 0; gq < 4; ++gq)
            *reinterpret_cast<float4*>(bt + t * LDF + 32 * wave + 8 * gq + 4 * half) =
                float4{wd[4 * gq] + add[4 * gq], wd[4 * gq + 1] + add[4 * gq + 1], wd[4 * gq + 2] + add[4 * gq + 2],
                       wd[4 * gq + 3] + add[4 * gq + 3]};
        __syncthreads();
        _Pragma("unroll") for (int it = 0; it < 4; ++it) {
            const int p = tid + NT * it, row = p >> 5, c4 = p & 31;
            if (row < L)
                *reinterpret_cast<float4*>(dg + (tok0 + size_t(row) * ts) * D + 4 * c4) = *reinterpret_cast<const float4*>(bt + row * LDF + 4 * c4);
        }
    }
}
