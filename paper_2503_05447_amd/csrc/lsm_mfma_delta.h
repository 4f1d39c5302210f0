// Delta-rule rows of the paper's Table 1 (DeltaNet, Gated DeltaNet), forward, chunkwise: bf16 operands, fp32
// accumulation, chunk = 64, d_k = d_v = 128.  Included by lsm_mfma.hip after lsm_mfma_walk.h.
//
// Both rows are  M_t = alpha_t (I - beta_t k_t^T k_t) M_{t-1} + b_t k_t^T v_t ,  o_t = q_t M_t  (DeltaNet:
// alpha = 1, beta = the row's a_t; Gated DeltaNet: alpha = the row's a_t, beta = 1).  With the pseudo-value
//     u_t = b_t v_t - alpha_t beta_t k_t M_{t-1}
// the update reads M_t = alpha_t M_{t-1} + k_t^T u_t: the per-token scalar-decay recurrence of Eq. 5 with u in
// the place of v, which the chunk walker already evaluates.  Inside a chunk that starts from the state S, with
// Gamma_t = prod_{s <= t} alpha_s, the pseudo-values solve the unit lower-triangular system
//     (I + L) U = diag(b) V - diag(beta Gamma) K S ,   L_tr = beta_t (Gamma_t / Gamma_r) (k_t . k_r) ,  r < t
// so U = Uhat - What S with  T = (I + L)^-1 ,  Uhat = T diag(b) V ,  What = T diag(beta Gamma) K  (the chunkwise
// form published for the delta rule; the paper itself gives no algorithm for these rows).
//   mk_delta_prep  (one workgroup per chunk, all chunks in parallel): L from K K^T on the matrix cores, T by
//                  forward substitution in fp32 inside 32 x 32 diagonal blocks and a block product below them,
//                  Uhat (fp32) and What (bf16) to the workspace.
//   mk_delta_walk  (one workgroup per sequence): the forward chunk walker with one more product per chunk,
//                  U = Uhat - What S from the state in the accumulators; U (as bf16 head + remainder) then plays the
//                  value tile's part in the intra-chunk product and in the state update.
// Every value column of the state evolves on its own (the erase term acts on the key side only), so a wave
// keeps its 128 x 32 slice of S and its 32 columns of U to itself.
// A sequence is walked by one workgroup from end to end: the state a segment would start from is not a decayed
// sum here (it carries the product of the erase factors), so the walkers' segment summaries do not apply.
#pragma once

constexpr int LDU = D + 4;   // floats per row of an fp32 [64][128] tile in LDS
constexpr int LDD = 36;      // floats per row of a 32 x 32 diagonal block of L
constexpr int LDT = 40;      // elements per row of a 32 x 32 bf16 tile
// LDS of mk_delta_prep (two workgroups per compute unit):
//   K tile | R1: the four planes of T^T scaled by columns (64 x LDP bf16 each), later the Uhat stage (fp32)
//          | R2: diagonal blocks of L (fp32; later R^T head, remainder), L_10 head, remainder, T_00^T and T_11^T head,
//                remainder (32 x LDT bf16 each); later the V tile
//          | log Gamma, beta, b
constexpr int kDeltaR1 = 4 * C * LDP * 2;
constexpr int kDeltaR2 = 2 * 32 * LDD * 4 + 6 * 32 * LDT * 2;
static_assert(kDeltaR1 >= C * LDU * 4 && kDeltaR2 >= C * LD * 2 && 2 * 32 * LDD * 4 >= 2 * 32 * LDT * 2, "tenants fit");
constexpr int kDeltaPrepLds = C * LD * 2 + kDeltaR1 + kDeltaR2 + 3 * C * 4;

struct DeltaPrepArgs {
    const uint16_t *k, *v;
    const float *log_alpha, *beta, *bw;  // per token ([B,H,T], or [B,T,H] for the token-major layout); NULL = 1
    uint16_t* what;                      // [BH*T][128] bf16
    float* uhat;                         // [BH*T][128] fp32
};

// 32 consecutive fp32 values -> one 32-element bf16 row, head and remainder
__device__ __forceinline__ void delta_row_split(uint16_t* hi, uint16_t* lo, const float (&x)[32], float scale) {
    _Pragma("unroll") for (int i = 0; i < 4; ++i) {
        u32x4 h, l;
        _Pragma("unroll") for (int p = 0; p < 4; ++p) {
            const float x0 = x[8 * i + 2 * p] * scale, x1 = x[8 * i + 2 * p + 1] * scale;
            h[p] = pack2(x0, x1);
            l[p] = pack2(x0 - bf16_lo(h[p]), x1 - bf16_hi(h[p]));
        }
        *reinterpret_cast<u32x4*>(hi + 8 * i) = h;
        *reinterpret_cast<u32x4*>(lo + 8 * i) = l;
    }
}

// grid: (N, BH).  T = (I + L)^-1 in two levels: the two 32 x 32 diagonal blocks by forward substitution in fp32
// (one wave, lane = block and column), the block below the diagonal as T_10 = -T_11 L_10 T_00 on the matrix cores
// with every factor as bf16 head + remainder.  T is kept transposed and already scaled by columns (b_r for Uhat,
// beta_r Gamma_r for What), so every lane writes whole 16-byte row pieces.
template <bool DEC>
__global__ __launch_bounds__(kThreads, 2) void mk_delta_prep(Dims d, DeltaPrepArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    uint16_t* Kt = reinterpret_cast<uint16_t*>(smem);
    unsigned char* r1 = reinterpret_cast<unsigned char*>(Kt + C * LD);
    uint16_t* TbTh = reinterpret_cast<uint16_t*>(r1);  // (T diag(b))^T [r][t], head and remainder
    uint16_t* TbTl = TbTh + C * LDP;
    uint16_t* TwTh = TbTl + C * LDP;                   // (T diag(beta Gamma))^T
    uint16_t* TwTl = TwTh + C * LDP;
    float* Ust = reinterpret_cast<float*>(r1);
    unsigned char* r2 = r1 + kDeltaR1;
    float* Ld = reinterpret_cast<float*>(r2);                              // [2][32][LDD]: L_00, L_11
    uint16_t* RTh = reinterpret_cast<uint16_t*>(r2);                       // over L_00, L_11 once they are spent
    uint16_t* RTl = RTh + 32 * LDT;
    uint16_t* L10h = reinterpret_cast<uint16_t*>(r2 + 2 * 32 * LDD * 4);   // L_10 [t'][r]
    uint16_t* L10l = L10h + 32 * LDT;
    uint16_t* TTh = L10l + 32 * LDT;                                       // [2] x (head, remainder): T_00^T, T_11^T, [c][t']
    uint16_t* Vt = reinterpret_cast<uint16_t*>(r2);
    float* lg = reinterpret_cast<float*>(r2 + kDeltaR2);  // log Gamma_t
    float* be = lg + C;
    float* bb = be + C;

    const int c = blockIdx.x, bh = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, n = lane & 31, half = lane >> 5;
    const ChunkPos cp = chunk_pos(d, c, bh);
    const int L = cp.L;
    if (L <= 0) return;
    if (wave == 0) {
        const size_t ptok = cp.tok0 + size_t(min(lane, L - 1)) * cp.ts;
        float x = (DEC && lane < L) ? a.log_alpha[ptok] : 0.f;
        const float bet = a.beta ? a.beta[ptok] : 1.f, bwt = a.bw ? a.bw[ptok] : 1.f;
        for (int off = 1; off < 64; off <<= 1) {
            const float y = __shfl_up(x, off, 64);
            if (lane >= off) x += y;
        }
        lg[lane] = x;
        be[lane] = lane < L ? bet : 0.f;  // rows beyond the ragged end: no erase, no write
        bb[lane] = lane < L ? bwt : 0.f;
    }
    TileRegs rv;
    tile_gload(rv, a.v, cp.tok0, cp.ts, L, tid);  // held in registers until the solve has freed its LDS
    load_tile(Kt, a.k, cp.tok0, cp.ts, L, tid);
    __syncthreads();
    // ---- L[t][r] = beta_t e^{lg_t - lg_r} (k_t . k_r) for r < t, else 0: blocks (r, t) = (0,0), (0,1), (1,1)
    if (wave < 3) {
        const int rb = wave == 2 ? 1 : 0, tb = wave ? 1 : 0;
        f32x16 G = score_block2(Kt, 32 * rb, Kt, 32 * tb, n, half);  // D[m = r][n = t]
        const int t = 32 * tb + n;
        const float bt = be[t], lt = lg[t];
        _Pragma("unroll") for (int g = 0; g < 4; ++g) {
            const float4 lr = *reinterpret_cast<const float4*>(lg + 32 * rb + 8 * g + 4 * half);
            const float lrv[4] = {lr.x, lr.y, lr.z, lr.w};
            _Pragma("unroll") for (int j = 0; j < 4; ++j) {
                const int r = 32 * rb + 8 * g + 4 * half + j;
                G[4 * g + j] = r < t ? bt * (DEC ? __expf(lt - lrv[j]) : 1.f) * G[4 * g + j] : 0.f;
            }
        }
        if (rb == tb) {  // diagonal block, fp32 [t'][r']
            float* dst = Ld + rb * 32 * LDD + n * LDD;
            _Pragma("unroll") for (int g = 0; g < 4; ++g)
                *reinterpret_cast<float4*>(dst + 8 * g + 4 * half) = float4{G[4 * g], G[4 * g + 1], G[4 * g + 2], G[4 * g + 3]};
        } else {         // L_10 [t'][r], bf16 head + remainder
            store_block_t_split(L10h, L10l, LDT, n, 0, half, G);
        }
    }
    __syncthreads();
    if (wave == 0) {
        // ---- diagonal blocks: X[t'] = [t' == c] - sum_{r' < t'} L_bb[t'][r'] X[r'], lane = (block, column c)
        const int blk = half, cc = n;
        const float* Lb = Ld + blk * 32 * LDD;
        float X[32];
        _Pragma("unroll") for (int t = 0; t < 32; ++t) X[t] = 0.f;
        _Pragma("unroll") for (int t = 0; t < 32; ++t) {
            float acc[4] = {cc == t ? 1.f : 0.f, 0.f, 0.f, 0.f};
            _Pragma("unroll") for (int q4 = 0; q4 < (t + 3) / 4; ++q4) {
                const float4 l = *reinterpret_cast<const float4*>(Lb + t * LDD + 4 * q4);
                acc[0] -= l.x * X[4 * q4];
                acc[1] -= l.y * X[4 * q4 + 1];
                acc[2] -= l.z * X[4 * q4 + 2];
                acc[3] -= l.w * X[4 * q4 + 3];
            }
            X[t] = (acc[0] + acc[1]) + (acc[2] + acc[3]);
        }
        const float bcol = bb[lane], wcol = be[lane] * (DEC ? __expf(lg[lane]) : 1.f);  // lane = this column's token
        uint16_t* tt = TTh + blk * 2 * 32 * LDT;
        delta_row_split(tt + cc * LDT, tt + 32 * LDT + cc * LDT, X, 1.f);
        delta_row_split(TbTh + lane * LDP + 32 * blk, TbTl + lane * LDP + 32 * blk, X, bcol);
        delta_row_split(TwTh + lane * LDP + 32 * blk, TwTl + lane * LDP + 32 * blk, X, wcol);
        __builtin_amdgcn_wave_barrier();  // LDS serves one wave's accesses in order: what follows reads what was just written
        // ---- R[r][t] = sum_t' L_10[t'][r] T_11[t][t'], kept as R^T [t][r]
        const uint16_t *T00h = TTh, *T00l = TTh + 32 * LDT, *T11h = TTh + 2 * 32 * LDT, *T11l = TTh + 3 * 32 * LDT;
        f32x16 R = {0};
        _Pragma("unroll") for (int ks = 0; ks < 2; ++ks) {
            const bf16x8 ah = frag_tr(L10h, LDT, 16 * ks, 0, lane), al = frag_tr(L10l, LDT, 16 * ks, 0, lane);
            const bf16x8 bh_ = frag_tr(T11h, LDT, 16 * ks, 0, lane), bl = frag_tr(T11l, LDT, 16 * ks, 0, lane);
            R = mfma(ah, bh_, R);
            R = mfma(ah, bl, R);
            R = mfma(al, bh_, R);
        }
        __builtin_amdgcn_wave_barrier();
        store_block_t_split(RTh, RTl, LDT, n, 0, half, R);  // over the diagonal blocks of L, which are spent
        __builtin_amdgcn_wave_barrier();
        // ---- T_10[t][c] = -sum_r R^T[t][r] T_00[r][c], scaled by this lane's column and stored transposed
        f32x16 T10 = {0};
        _Pragma("unroll") for (int ks = 0; ks < 2; ++ks) {
            const bf16x8 ah = frag(RTh, LDT, n, 16 * ks + 8 * half), al = frag(RTl, LDT, n, 16 * ks + 8 * half);
            const bf16x8 bh_ = frag(T00h, LDT, n, 16 * ks + 8 * half), bl = frag(T00l, LDT, n, 16 * ks + 8 * half);
            T10 = mfma(ah, bh_, T10);
            T10 = mfma(ah, bl, T10);
            T10 = mfma(al, bh_, T10);
        }
        const float b0 = bb[n], w0 = be[n] * (DEC ? __expf(lg[n]) : 1.f);  // column c = n of the first block
        f32x16 Tb, Tw;
        _Pragma("unroll") for (int x = 0; x < 16; ++x) {
            Tb[x] = -T10[x] * b0;
            Tw[x] = -T10[x] * w0;
        }
        store_block_t_split(TbTh, TbTl, LDP, n, 32, half, Tb);  // rows c, columns 32 + t
        store_block_t_split(TwTh, TwTl, LDP, n, 32, half, Tw);
    }
    __syncthreads();  // T is complete; the small tiles are spent
    tile_commit(Vt, rv, L, tid);
    __syncthreads();
    // ---- What^T[c][t] = sum_r K[r][c] Tw[t][r],  Uhat^T[c][t] = sum_r V[r][c] Tb[t][r]; this wave: features 32 w ..
    f32x16 Wt[2] = {{0}, {0}}, Ut[2] = {{0}, {0}};
    _Pragma("unroll") for (int nb = 0; nb < 2; ++nb)
        _Pragma("unroll") for (int ks = 0; ks < 2 * (nb + 1); ++ks) {  // T is lower triangular
            const bf16x8 ka = frag_tr(Kt, LD, 16 * ks, 32 * wave, lane), va = frag_tr(Vt, LD, 16 * ks, 32 * wave, lane);
            Wt[nb] = mfma(ka, frag_tr(TwTh, LDP, 16 * ks, 32 * nb, lane), Wt[nb]);
            Wt[nb] = mfma(ka, frag_tr(TwTl, LDP, 16 * ks, 32 * nb, lane), Wt[nb]);
            Ut[nb] = mfma(va, frag_tr(TbTh, LDP, 16 * ks, 32 * nb, lane), Ut[nb]);
            Ut[nb] = mfma(va, frag_tr(TbTl, LDP, 16 * ks, 32 * nb, lane), Ut[nb]);
        }
    __syncthreads();  // every read of the tiles and of the planes is done
    _Pragma("unroll") for (int nb = 0; nb < 2; ++nb) {
        store_packed(Kt, LD, 32 * nb + n, 32 * wave, half, pack_block(Wt[nb]));
        _Pragma("unroll") for (int g = 0; g < 4; ++g)
            *reinterpret_cast<float4*>(Ust + (32 * nb + n) * LDU + 32 * wave + 8 * g + 4 * half) =
                float4{Ut[nb][4 * g], Ut[nb][4 * g + 1], Ut[nb][4 * g + 2], Ut[nb][4 * g + 3]};
    }
    __syncthreads();
    _Pragma("unroll") for (int it = 0; it < 4; ++it) {
        const int p = tid + kThreads * it, row = p >> 4, cpp = p & 15;
        if (row < L)
            *reinterpret_cast<u32x4*>(a.what + (cp.wtok0 + row) * D + cpp * 8) = *reinterpret_cast<const u32x4*>(Kt + row * LD + cpp * 8);
    }
    _Pragma("unroll") for (int it = 0; it < 8; ++it) {
        const int p = tid + kThreads * it, row = p >> 5, c4 = p & 31;
        if (row < L)
            *reinterpret_cast<float4*>(a.uhat + (cp.wtok0 + row) * D + c4 * 4) = *reinterpret_cast<const float4*>(Ust + row * LDU + c4 * 4);
    }
}

// ---- the walker
struct DeltaWalkArgs {
    const uint16_t *q, *k;
    const uint16_t* what;   // [BH*T][128]
    const float* uhat;      // [BH*T][128]
    const float* log_alpha;
    uint16_t* out;
    const float* edge_in;   // M_0 [i][v] per sequence or NULL
    float* edge_out;        // M_T or NULL
};
// LDS: Q | K | U head (the value tile's place) | U remainder | What (64 x LD bf16 each) | Uhat (64 x LDU fp32) |
// scores head | scores remainder (64 x LDP) | bs | wo
constexpr int kDeltaWalkLds = (5 * C * LD + 2 * C * LDP) * 2 + C * LDU * 4 + (2 * C + 8) * 4;

// The pseudo-values are kept as bf16 head + remainder: a single rounding of u_t would show in o_t at the size of
// an output ulp wherever one token dominates the read-out (strong decay), which the diagonal kinds never pay
// because their values are inputs.
// intra: O^T[v][j] += sum_{r <= j} U^T[v][r] P[j][r] for the query block jb (remainder x remainder left out)
__device__ __forceinline__ void delta_intra(f32x16& O, int jb, const uint16_t* Vh, const uint16_t* Vl, const uint16_t* Ph,
                                            const uint16_t* Pl, int w4, int lane, int n, int half) {
    const int j = 32 * jb + n;
    _Pragma("unroll") for (int ks = 0; ks < 4; ++ks) {
        if (ks >= 2 * (jb + 1)) break;  // keys r >= 32 never reach queries j < 32
        const bf16x8 vh = frag_tr(Vh, LD, 16 * ks, 32 * w4, lane), vl = frag_tr(Vl, LD, 16 * ks, 32 * w4, lane);
        const bf16x8 ph = frag(Ph, LDP, j, 16 * ks + 8 * half);
        O = mfma(vh, ph, O);
        O = mfma(vl, ph, O);
        O = mfma(vh, frag(Pl, LDP, j, 16 * ks + 8 * half), O);
    }
}
// state: S[i][v] = e^{b_C} S[i][v] + sum_t K^T[i][t] (wo_t U[t][v]), U from its two planes, the weighted slice split
// again into head + remainder in registers
template <bool DEC>
__device__ __forceinline__ void delta_update(f32x16 (&S)[4], const uint16_t* K, const uint16_t* Vh, const uint16_t* Vl,
                                             const float* wo, float bC, int w4, int lane, int half) {
    if (DEC) {
        const float lam = __expf(bC);
        _Pragma("unroll") for (int ib = 0; ib < 4; ++ib)
            _Pragma("unroll") for (int x = 0; x < 16; ++x) S[ib][x] *= lam;
    }
    _Pragma("unroll") for (int ks = 0; ks < 4; ++ks) {
        const u32x4 rh = __builtin_bit_cast(u32x4, frag_tr(Vh, LD, 16 * ks, 32 * w4, lane));
        const u32x4 rl = __builtin_bit_cast(u32x4, frag_tr(Vl, LD, 16 * ks, 32 * w4, lane));
        u32x4 hi = rh, lo = rl;
        if (DEC) {
            const float4 w0 = *reinterpret_cast<const float4*>(wo + 16 * ks + 8 * half);
            const float4 w1 = *reinterpret_cast<const float4*>(wo + 16 * ks + 8 * half + 4);
            const float w[8] = {w0.x, w0.y, w0.z, w0.w, w1.x, w1.y, w1.z, w1.w};
            _Pragma("unroll") for (int p = 0; p < 4; ++p) {
                const float x0 = (bf16_lo(rh[p]) + bf16_lo(rl[p])) * w[2 * p], x1 = (bf16_hi(rh[p]) + bf16_hi(rl[p])) * w[2 * p + 1];
                hi[p] = pack2(x0, x1);
                lo[p] = pack2(x0 - bf16_lo(hi[p]), x1 - bf16_hi(hi[p]));
            }
        }
        const bf16x8 vh = __builtin_bit_cast(bf16x8, hi), vl = __builtin_bit_cast(bf16x8, lo);
        bf16x8 ka[4];
        _Pragma("unroll") for (int ib = 0; ib < 4; ++ib) ka[ib] = frag_tr(K, LD, 16 * ks, 32 * ib, lane);
        _Pragma("unroll") for (int ib = 0; ib < 4; ++ib) S[ib] = mfma(ka[ib], vh, S[ib]);
        _Pragma("unroll") for (int ib = 0; ib < 4; ++ib) S[ib] = mfma(ka[ib], vl, S[ib]);
    }
}

struct TileRegsF { float4 v[8]; };
__device__ __forceinline__ void tilef_gload(TileRegsF& r, const float* src, size_t tok0, int L, int tid) {
    _Pragma("unroll") for (int it = 0; it < 8; ++it) {
        const int p = tid + kThreads * it, row = min(p >> 5, L - 1), c4 = p & 31;
        r.v[it] = *reinterpret_cast<const float4*>(src + (tok0 + row) * D + c4 * 4);
    }
}
__device__ __forceinline__ void tilef_commit(float* dst, const TileRegsF& r, int L, int tid) {
    _Pragma("unroll") for (int it = 0; it < 8; ++it) {
        const int p = tid + kThreads * it, row = p >> 5, c4 = p & 31;
        const float keep = row < L ? 1.f : 0.f;
        *reinterpret_cast<float4*>(dst + row * LDU + c4 * 4) = float4{r.v[it].x * keep, r.v[it].y * keep, r.v[it].z * keep, r.v[it].w * keep};
    }
}

// grid: (seqs)
template <bool DEC>
__global__ __launch_bounds__(kThreads, 1) void mk_delta_walk(Dims d, DeltaWalkArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    uint16_t* Q = reinterpret_cast<uint16_t*>(smem);
    uint16_t* K = Q + C * LD;
    uint16_t* V = K + C * LD;    // pseudo-values U of this chunk, bf16 head
    uint16_t* Vl = V + C * LD;   // and remainder
    uint16_t* Wh = Vl + C * LD;
    float* Uh = reinterpret_cast<float*>(Wh + C * LD);
    uint16_t* Ph = reinterpret_cast<uint16_t*>(Uh + C * LDU);
    uint16_t* Pl = Ph + C * LDP;
    float* bs = reinterpret_cast<float*>(Pl + C * LDP);
    float* wo = bs + C + 4;
    uint16_t* stage = Q;

    const int seq = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, n = lane & 31, half = lane >> 5;
    const SeqWalk walk = seq_walk(d, seq);
    const int cnt = walk.n;

    f32x16 S[4];
    _Pragma("unroll") for (int ib = 0; ib < 4; ++ib) S[ib] = f32x16{0};
    if (a.edge_in) walk_state_load(S, a.edge_in + size_t(seq) * D * D, false, wave, n, half);

    TileRegs rq, rk, rw;
    TileRegsF ru;
    float gval = 0.f;
    auto gload = [&](int kk) {
        const ChunkPos p = walk_pos(d, walk, min(kk, cnt - 1));
        if (DEC) gval = a.log_alpha[p.tok0 + size_t(min(lane, p.L - 1)) * p.ts];
        walk_gload<false, kThreads>(rq, a.q, p.tok0, p.ts, p.L, tid);
        walk_gload<false, kThreads>(rk, a.k, p.tok0, p.ts, p.L, tid);
        walk_gload<false, kThreads>(rw, a.what, p.wtok0, 1, p.L, tid);
        tilef_gload(ru, a.uhat, p.wtok0, p.L, tid);
    };
    if (cnt > 0) gload(0);

    for (int kk = 0; kk < cnt; ++kk) {
        const ChunkPos cp = walk_pos(d, walk, kk);
        const int L = cp.L;
        walk_commit<kThreads>(Q, rq, L, tid);
        walk_commit<kThreads>(K, rk, L, tid);
        walk_commit<kThreads>(Wh, rw, L, tid);
        tilef_commit(Uh, ru, L, tid);
        if (DEC && wave == 0) walk_decay_tables<false>(gval, L, 0.f, bs, wo, lane);
        gload(kk + 1);
        __syncthreads();  // (A) tiles and decay tables of this chunk are in LDS
        const float bC = DEC ? bs[C] : 0.f;

        // pseudo-values of this wave's value columns: U^T[v][t] = Uhat[t][v] - sum_i S[i][v] What[t][i]
        {
            f32x16 Wacc[2];
            walk_inter<false>(Wacc, S, Wh, bs, n, half);
            _Pragma("unroll") for (int tb = 0; tb < 2; ++tb) {
                f32x16 u;
                _Pragma("unroll") for (int g = 0; g < 4; ++g) {
                    const float4 uh = *reinterpret_cast<const float4*>(Uh + (32 * tb + n) * LDU + 32 * wave + 8 * g + 4 * half);
                    u[4 * g + 0] = uh.x - Wacc[tb][4 * g + 0];
                    u[4 * g + 1] = uh.y - Wacc[tb][4 * g + 1];
                    u[4 * g + 2] = uh.z - Wacc[tb][4 * g + 2];
                    u[4 * g + 3] = uh.w - Wacc[tb][4 * g + 3];
                }
                const PackedBlock uh = pack_block(u);
                _Pragma("unroll") for (int g = 0; g < 4; ++g) {
                    u[4 * g + 0] -= bf16_lo(uh.v[g].x);
                    u[4 * g + 1] -= bf16_hi(uh.v[g].x);
                    u[4 * g + 2] -= bf16_lo(uh.v[g].y);
                    u[4 * g + 3] -= bf16_hi(uh.v[g].y);
                }
                store_packed(V, LD, 32 * tb + n, 32 * wave, half, uh);
                store_packed(Vl, LD, 32 * tb + n, 32 * wave, half, pack_block(u));
            }
        }
        f32x16 O[2];
        walk_inter<DEC>(O, S, Q, bs, n, half);
        walk_scores<DEC>(K, Q, Ph, Pl, bs, wave, n, half);
        __syncthreads();  // (C) scores are in LDS; nobody reads Q any more (this wave's columns of U are its own)
        _Pragma("unroll") for (int jb = 0; jb < 2; ++jb) {
            delta_intra(O[jb], jb, V, Vl, Ph, Pl, wave, lane, n, half);
            store_packed(stage, LD, 32 * jb + n, 32 * wave, half, pack_block(O[jb]));
        }
        delta_update<DEC>(S, K, V, Vl, wo, bC, wave, lane, half);
        __syncthreads();  // (D) the output stage is complete and every read of this chunk's tiles is done
        walk_store<false>(a.out, stage, cp.tok0, cp.ts, L, tid);
    }
    if (a.edge_out) walk_state_store(S, a.edge_out + size_t(seq) * D * D, false, wave, n, half);
}
