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
//   mk_delta_walk8 (one workgroup per sequence or segment): the forward chunk walker with one more product per chunk,
//                  U = Uhat - What S from the state in the accumulators; U (as bf16 head + remainder) then plays the
//                  value tile's part in the intra-chunk product and in the state update.
// Every value column of the state evolves on its own (the erase term acts on the key side only), so a wave
// keeps its 128 x 32 slice of S and its 32 columns of U to itself.
// Segments.  The state a segment of chunks ends with is an affine function of the state it starts from, S' = A S + B,
// with a dense d_k x d_k factor A (the product of the chunks' erase-and-decay factors), not a decayed sum.  Because
// the value columns evolve independently, A is what the same walk makes of the identity when the values are zero,
// and B what it makes of a zero state: with fewer sequences than compute units, a summary pass runs the state part
// of the walker twice per segment (MODE 1: B, MODE 2: A), mk_delta_combine chains E' = A E + B over the segments of
// each sequence on the matrix cores, and the walker proper then runs all segments in parallel.
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
    uint16_t* tt;                        // NULL, or [BH*N][2][64][64] bf16: T^T (rows r, columns t), head and remainder planes
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

    const int c = blockIdx.x, bh = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), n = lane & 31, half = lane >> 5;
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
        uint16_t* gtt = a.tt ? a.tt + cp.slot * 2 * C * C : nullptr;  // the backward pass wants T itself
        if (gtt) {
            delta_row_split(gtt + lane * C + 32 * blk, gtt + C * C + lane * C + 32 * blk, X, 1.f);
            if (blk) {  // T[t][r] = 0 for t < 32 <= r
                _Pragma("unroll") for (int i = 0; i < 4; ++i) {
                    *reinterpret_cast<u32x4*>(gtt + lane * C + 8 * i) = u32x4{0, 0, 0, 0};
                    *reinterpret_cast<u32x4*>(gtt + C * C + lane * C + 8 * i) = u32x4{0, 0, 0, 0};
                }
            }
        }
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
        if (gtt) {
            _Pragma("unroll") for (int x = 0; x < 16; ++x) Tb[x] = -T10[x];
            store_block_t_split(gtt, gtt + C * C, C, n, 32, half, Tb);
        }
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
    uint16_t *usave, *usave_l;  // NULL, or the pseudo-values (bf16 head, remainder) in the layout of v, for the backward pass
    // segments (nseg > 1): m chunks each; the walker enters segment s with bound[seq][s]; the summary modes leave their
    // end state in sum[seq][s] ([i][v] fp32, 128 x 128 each)
    int m, nseg;
    const float* bound;
    float* sum;
};
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

// The walk (MODE 0), and the summaries of a segment for the cut into segments: the state part of the walk alone, from a
// zero state (MODE 1: the segment's own contribution B) or from the identity with zero values (MODE 2: its transfer
// matrix A).  grid: (segments, seqs).  Eight waves, two per SIMD, split by function:
//   waves 0..3 carry the state (wave w: value columns [32w, 32w+32)): both inter products, the pseudo-values, the intra
//              part of the output and the state update - the chain that every chunk has to go through in order;
//   waves 4..7 do everything that does not need the state: all tile traffic (global -> registers -> LDS one chunk ahead,
//              output stage and pseudo-values -> global), the decay tables, the three score blocks.
// A chunk has two phases.  In the first the carrier waves read Q, What and Uhat (inter products, pseudo-values) while the
// others compute the scores and store the previous chunk's output; in the second the carrier waves read only the scores,
// K and their own pseudo-values (intra part, state update), so the others overwrite Q, What and Uhat with the next
// chunk's rows and rebuild the decay tables (two sets, used in turn) meanwhile.  Only K, which both phases read, is
// committed between two chunks.  The output has a stage of its own for the same reason.
// LDS: Q | K | U head | U remainder | What | output stage (64 x LD bf16 each) | Uhat (64 x LDU fp32) | scores head |
// scores remainder (64 x LDP) | two sets of (bs, wo)
constexpr int kDeltaTab = 2 * C + 8;
constexpr int kDeltaWalk8Lds = (6 * C * LD + 2 * C * LDP) * 2 + C * LDU * 4 + 2 * kDeltaTab * 4;
static_assert(kDeltaWalk8Lds <= 160 * 1024, "one workgroup's LDS");

template <bool DEC, int MODE>
__global__ __launch_bounds__(512, 1) void mk_delta_walk8(Dims d, DeltaWalkArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    uint16_t* Q = reinterpret_cast<uint16_t*>(smem);
    uint16_t* K = Q + C * LD;
    uint16_t* V = K + C * LD;    // pseudo-values U of this chunk, bf16 head
    uint16_t* Vl = V + C * LD;   // and remainder
    uint16_t* Wh = Vl + C * LD;
    uint16_t* stage = Wh + C * LD;
    float* Uh = reinterpret_cast<float*>(stage + C * LD);
    uint16_t* Ph = reinterpret_cast<uint16_t*>(Uh + C * LDU);
    uint16_t* Pl = Ph + C * LDP;
    float* tab = reinterpret_cast<float*>(Pl + C * LDP);  // [2][kDeltaTab]: bs (65), wo (64) of the chunks of either parity

    // the wave index as a scalar: the branch between the two groups is a scalar branch
    const int seg = blockIdx.x, seq = blockIdx.y, tid = threadIdx.x, wave8 = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63, wave = wave8 & 3, n = lane & 31, half = lane >> 5;
    const int t256 = tid & 255;
    const bool carrier = wave8 < 4;
    const SeqWalk walk = seq_walk(d, seq);
    const int nsq = max(1, (walk.n + a.m - 1) / a.m);  // segments of this sequence
    const int kbeg = seg * a.m, kend = min(walk.n, kbeg + a.m), cnt = max(kend - kbeg, 0);
    if (MODE != 0) {
        if (cnt <= 0 || seg >= nsq - 1) return;  // only segments whose end state another one starts from
    } else if (seg >= nsq) {
        return;
    }

    if (carrier) {
        f32x16 S[4];
        _Pragma("unroll") for (int ib = 0; ib < 4; ++ib) S[ib] = f32x16{0};
        if (MODE == 0) {
            const float* ein = a.nseg > 1 ? a.bound + (size_t(seq) * a.nseg + seg) * D * D
                                          : (a.edge_in ? a.edge_in + size_t(seq) * D * D : nullptr);
            if (ein) walk_state_load(S, ein, false, wave, n, half);
        } else if (MODE == 2) {
            _Pragma("unroll") for (int ib = 0; ib < 4; ++ib)
                _Pragma("unroll") for (int x = 0; x < 16; ++x)
                    S[ib][x] = (32 * ib + 8 * (x >> 2) + 4 * half + (x & 3) == 32 * wave + n) ? 1.f : 0.f;
        }
        for (int kk = 0; kk < cnt; ++kk) {
            const float* bs = tab + (kk & 1) * kDeltaTab;
            const float* wo = bs + C + 4;
            __syncthreads();  // (A) the tiles and the decay tables of this chunk are in LDS
            const float bC = DEC ? bs[C] : 0.f;
            // pseudo-values of this wave's value columns: U^T[v][t] = Uhat[t][v] - sum_i S[i][v] What[t][i]; the inter part
            // of the output comes out of the same pass over the state blocks (one conversion to bf16 head + remainder)
            f32x16 O[2];
            {
                f32x16 Wacc[2];
                walk_inter_pair<DEC, MODE == 0>(Wacc, O, S, Wh, Q, bs, n, half);
                _Pragma("unroll") for (int tb = 0; tb < 2; ++tb) {
                    f32x16 u;
                    _Pragma("unroll") for (int g = 0; g < 4; ++g) {
                        const float4 uh = MODE == 2 ? float4{0.f, 0.f, 0.f, 0.f}
                                                    : *reinterpret_cast<const float4*>(Uh + (32 * tb + n) * LDU + 32 * wave + 8 * g + 4 * half);
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
            __syncthreads();  // (C) scores are in LDS; Q, What and Uhat are spent (this wave's columns of U are its own)
            if (MODE == 0) {
                _Pragma("unroll") for (int jb = 0; jb < 2; ++jb) {
                    delta_intra(O[jb], jb, V, Vl, Ph, Pl, wave, lane, n, half);
                    store_packed(stage, LD, 32 * jb + n, 32 * wave, half, pack_block(O[jb]));
                }
            }
            walk_update_vsplit<DEC, true>(S, K, V, Vl, wo, bC, wave, lane, half);
            __syncthreads();  // (D) the output stage is complete and every read of K and of the pseudo-values is done
        }
        if (MODE != 0) walk_state_store(S, a.sum + (size_t(seq) * a.nseg + seg) * D * D, false, wave, n, half);
        else if (a.edge_out && seg == nsq - 1) walk_state_store(S, a.edge_out + size_t(seq) * D * D, false, wave, n, half);
    } else {
        TileRegs rq, rk, rw;
        TileRegsF ru;
        float gval = 0.f;
        auto pos = [&](int kk) { return walk_pos(d, walk, kbeg + min(kk, cnt - 1)); };
        auto gload_main = [&](int kk) {  // the rows of the first phase, and the log-decays
            const ChunkPos p = pos(kk);
            if (DEC) gval = a.log_alpha[p.tok0 + size_t(min(lane, p.L - 1)) * p.ts];
            if (MODE == 0) walk_gload<false, kThreads>(rq, a.q, p.tok0, p.ts, p.L, t256);
            walk_gload<false, kThreads>(rw, a.what, p.wtok0, 1, p.L, t256);
            if (MODE != 2) tilef_gload(ru, a.uhat, p.wtok0, p.L, t256);
        };
        auto commit_main = [&](int kk) {  // ... into LDS, with the decay tables of that chunk
            const int L = pos(kk).L;
            if (MODE == 0) walk_commit<kThreads>(Q, rq, L, t256);
            walk_commit<kThreads>(Wh, rw, L, t256);
            if (MODE != 2) tilef_commit(Uh, ru, L, t256);
            float* bs = tab + (kk & 1) * kDeltaTab;
            if (DEC && wave == 0) walk_decay_tables<false>(gval, L, 0.f, bs, bs + C + 4, lane);
        };
        auto gload_k = [&](int kk) {
            const ChunkPos p = pos(kk);
            walk_gload<false, kThreads>(rk, a.k, p.tok0, p.ts, p.L, t256);
        };
        if (cnt > 0) {
            gload_main(0);
            gload_k(0);
            commit_main(0);
            if (cnt > 1) gload_main(1);
        }
        for (int kk = 0; kk < cnt; ++kk) {
            const ChunkPos cp = pos(kk);
            walk_commit<kThreads>(K, rk, cp.L, t256);
            __syncthreads();  // (A)
            if (kk + 1 < cnt) gload_k(kk + 1);
            if (MODE == 0) walk_scores<DEC>(K, Q, Ph, Pl, tab + (kk & 1) * kDeltaTab, wave, n, half);
            if (MODE == 0 && kk > 0 && a.out) {  // the previous chunk's output
                const ChunkPos pp = pos(kk - 1);
                walk_store<false, kThreads>(a.out, stage, pp.tok0, pp.ts, pp.L, t256);
            }
            __syncthreads();  // (C)
            if (kk + 1 < cnt) {
                commit_main(kk + 1);
                if (kk + 2 < cnt) gload_main(kk + 2);
            }
            if (MODE == 0 && a.usave) {
                walk_store<false, kThreads>(a.usave, V, cp.tok0, cp.ts, cp.L, t256);
                walk_store<false, kThreads>(a.usave_l, Vl, cp.tok0, cp.ts, cp.L, t256);
            }
            __syncthreads();  // (D)
        }
        if (MODE == 0 && cnt > 0 && a.out) {
            const ChunkPos pp = pos(cnt - 1);
            walk_store<false, kThreads>(a.out, stage, pp.tok0, pp.ts, pp.L, t256);
        }
    }
}

// Entry state of every segment: E_0 = M_0, E_{s+1} = A_s E_s + B_s (REV: from the last segment down, for the state
// gradients), one workgroup per sequence, the product on the
// matrix cores with both factors as bf16 head + remainder (three products; about 2^-16 relative).
// LDS: A head | A remainder | E head | E remainder (128 x LD each).   grid: (seqs)
constexpr int kDeltaCombineLds = 4 * D * LD * 2;
__device__ __forceinline__ void delta_split_tile(uint16_t* hi, uint16_t* lo, const float* src, int tid) {
    _Pragma("unroll") for (int it = 0; it < 16; ++it) {   // 128 x 128 floats by 256 threads, 4 at a time
        const int p = tid + kThreads * it, row = p >> 5, c4 = p & 31;
        const float4 x = src ? *reinterpret_cast<const float4*>(src + row * D + 4 * c4) : float4{0.f, 0.f, 0.f, 0.f};
        const uint32_t h0 = pack2(x.x, x.y), h1 = pack2(x.z, x.w);
        *reinterpret_cast<u32x2*>(hi + row * LD + 4 * c4) = u32x2{h0, h1};
        *reinterpret_cast<u32x2*>(lo + row * LD + 4 * c4) =
            u32x2{pack2(x.x - bf16_lo(h0), x.y - bf16_hi(h0)), pack2(x.z - bf16_lo(h1), x.w - bf16_hi(h1))};
    }
}
template <bool REV>
__global__ __launch_bounds__(kThreads, 1) void mk_delta_combine(Dims d, const float* __restrict__ edge_in, const float* __restrict__ sumA,
                                                                const float* __restrict__ sumB, float* __restrict__ bound, int m,
                                                                int nseg) {
    extern __shared__ __align__(16) unsigned char smem[];
    uint16_t* Ah = reinterpret_cast<uint16_t*>(smem);
    uint16_t* Al = Ah + D * LD;
    uint16_t* Eh = Al + D * LD;
    uint16_t* El = Eh + D * LD;
    const int seq = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), n = lane & 31, half = lane >> 5;
    const SeqWalk walk = seq_walk(d, seq);
    const int nsq = max(1, (walk.n + m - 1) / m);
    const float* e0 = edge_in ? edge_in + size_t(seq) * D * D : nullptr;
    float* b = bound + size_t(seq) * nseg * D * D;
    // the walk's first segment (REV: the last in time) starts from the edge state; the same as tiles
    float* b0 = b + size_t(REV ? nsq - 1 : 0) * D * D;
    _Pragma("unroll") for (int it = 0; it < 16; ++it) {
        const int p = tid + kThreads * it, row = p >> 5, c4 = p & 31;
        *reinterpret_cast<float4*>(b0 + row * D + 4 * c4) = e0 ? *reinterpret_cast<const float4*>(e0 + row * D + 4 * c4) : float4{0.f, 0.f, 0.f, 0.f};
    }
    delta_split_tile(Eh, El, e0, tid);
    for (int st = 0; st + 1 < nsq; ++st) {
        const int s = REV ? nsq - 1 - st : st;   // the segment walked in this step; its end state enters segment s -+ 1
        const size_t slot = (size_t(seq) * nseg + s) * D * D;
        delta_split_tile(Ah, Al, sumA + slot, tid);
        __syncthreads();  // A and E tiles are complete
        // E'[i][v] = sum_j A[i][j] E[j][v] + B[i][v]; this wave: rows i in [32 w, 32 w + 32)
        f32x16 acc[4];
        _Pragma("unroll") for (int vb = 0; vb < 4; ++vb)
            _Pragma("unroll") for (int x = 0; x < 16; ++x)
                acc[vb][x] = sumB[slot + size_t(32 * wave + 8 * (x >> 2) + 4 * half + (x & 3)) * D + 32 * vb + n];
        _Pragma("unroll") for (int ks = 0; ks < 8; ++ks) {
            const bf16x8 ah = frag(Ah, LD, 32 * wave + n, 16 * ks + 8 * half), al = frag(Al, LD, 32 * wave + n, 16 * ks + 8 * half);
            _Pragma("unroll") for (int vb = 0; vb < 4; ++vb) {
                const bf16x8 eh = frag_tr(Eh, LD, 16 * ks, 32 * vb, lane), el = frag_tr(El, LD, 16 * ks, 32 * vb, lane);
                acc[vb] = mfma(ah, eh, acc[vb]);
                acc[vb] = mfma(ah, el, acc[vb]);
                acc[vb] = mfma(al, eh, acc[vb]);
            }
        }
        __syncthreads();  // every wave has read E
        float* out = b + size_t(REV ? s - 1 : s + 1) * D * D;
        _Pragma("unroll") for (int vb = 0; vb < 4; ++vb)
            _Pragma("unroll") for (int x = 0; x < 16; ++x) {
                const int i = 32 * wave + 8 * (x >> 2) + 4 * half + (x & 3), v = 32 * vb + n;
                const float e = acc[vb][x];
                out[size_t(i) * D + v] = e;
                const uint32_t h = pack2(e, 0.f);
                Eh[i * LD + v] = uint16_t(h & 0xffffu);
                El[i * LD + v] = uint16_t(pack2(e - bf16_lo(h), 0.f) & 0xffffu);
            }
        // the next delta_split_tile writes A only; the barrier at the top of the next step orders the E writes
    }
}

// ---------------------------------------------------------------------------------------------
// Backward, sequential part.  With U known, M_t = alpha_t M_{t-1} + k_t^T u_t is the scalar-decay recurrence on values
// U, so the gradient walker of the diagonal kinds yields dq, the key gradient through the scores and the state
// update, and the decay gradient of those terms, PROVIDED it is handed the state gradients of the delta rule.  Those
// differ from the diagonal kinds': u_t depends on the state the chunk starts from (U = Uhat - What S), so per chunk
//     dU = A^T dO + diag(wo) K dS'          (A = masked decayed scores, dS' = gradient of the state at the chunk end)
//     dS = Gamma_C dS' + (diag(Gamma) Q)^T dO - What^T dU .
// mk_delta_rwalk walks a sequence backward with dS in the accumulators (the forward walker's block layout), stores
// dS' per chunk in the fragment-major bf16 form the gradient walker reads, and dU as bf16 head + remainder for the
// kernels that take the gradient through the triangular solve.  The gradient walker, which has the state S of
// every chunk in its accumulators, also forms dWhat = -dU S^T on the way (its VSPLIT variant).
struct DeltaRevArgs {
    const uint16_t *q, *k, *d_o;
    const uint16_t* what;     // [BH*T][128] bf16 (library order)
    const float* log_alpha;
    uint16_t* dstates;        // [BH*N] fragment-major bf16: slot c = gradient of the state at the end of chunk c
    uint16_t *du_h, *du_l;    // [BH*T][128] bf16 (library order)
    const float* edge_in;     // d M_T [i][v] per sequence or NULL
    float* edge_out;          // d M_0 or NULL
    int m, nseg;              // segments as for the forward walker: the walk enters segment s (from above) with bound[seq][s],
    const float* bound;       // the summary modes leave what the segment makes of a zero / identity state in sum[seq][s]
    float* sum;
};
constexpr int LDW = 40;  // row stride of a wave's private 32-column tiles
// LDS: Q | K | dO | What (64 x LD) | scores head | remainder (64 x LDP) | per wave: 128 x LDW bf16 (its columns of dS',
// then of dU head and remainder, 64 x LDW each) | bs | wo | Gamma
constexpr int kDeltaRevLds = (4 * C * LD + 2 * C * LDP) * 2 + 4 * D * LDW * 2 + (3 * C + 8) * 4;

// grid: (segments, seqs).  MODE 0: the walk.  MODE 1 / 2: summary of a segment (nothing stored but its end state), from a
// zero state / from the identity with d_o = 0.
template <bool DEC, int MODE = 0>
__global__ __launch_bounds__(kThreads, 1) void mk_delta_rwalk(Dims d, DeltaRevArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    uint16_t* Q = reinterpret_cast<uint16_t*>(smem);
    uint16_t* K = Q + C * LD;
    uint16_t* dO = K + C * LD;
    uint16_t* Wh = dO + C * LD;
    uint16_t* Ph = Wh + C * LD;
    uint16_t* Pl = Ph + C * LDP;
    uint16_t* priv = Pl + C * LDP;
    float* bs = reinterpret_cast<float*>(priv + 4 * D * LDW);
    float* wo = bs + C + 4;
    float* gm = wo + C + 4;

    const int seg = blockIdx.x, seq = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), n = lane & 31, half = lane >> 5;
    const SeqWalk walk = seq_walk(d, seq);
    const int nsq = max(1, (walk.n + a.m - 1) / a.m);
    const int kbeg = seg * a.m, kend = min(walk.n, kbeg + a.m), cnt = max(kend - kbeg, 0);
    if (MODE != 0) {
        if (cnt <= 0 || seg == 0) return;  // only segments whose end state (backward in time) another one starts from
    } else if (seg >= nsq) {
        return;
    }
    uint16_t* pw = priv + wave * D * LDW;   // this wave's region
    uint16_t* duh = pw;
    uint16_t* dul = pw + C * LDW;

    f32x16 S[4];  // dS[ib][4g+j] = dS[i = 32 ib + 8g + 4 half + j][v = 32 wave + n]
    _Pragma("unroll") for (int ib = 0; ib < 4; ++ib) S[ib] = f32x16{0};
    if (MODE == 0) {
        const float* ein = a.nseg > 1 ? a.bound + (size_t(seq) * a.nseg + seg) * D * D
                                      : (a.edge_in ? a.edge_in + size_t(seq) * D * D : nullptr);
        if (ein) walk_state_load(S, ein, false, wave, n, half);
    } else if (MODE == 2) {
        _Pragma("unroll") for (int ib = 0; ib < 4; ++ib)
            _Pragma("unroll") for (int x = 0; x < 16; ++x)
                S[ib][x] = (32 * ib + 8 * (x >> 2) + 4 * half + (x & 3) == 32 * wave + n) ? 1.f : 0.f;
    }

    TileRegs rq, rk, ro, rw;
    float gval = 0.f;
    auto gload = [&](int kk) {
        const ChunkPos p = walk_pos(d, walk, kend - 1 - min(kk, cnt - 1));
        if (DEC) gval = a.log_alpha[p.tok0 + size_t(min(lane, p.L - 1)) * p.ts];
        if (MODE != 2) {
            walk_gload<false, kThreads>(rq, a.q, p.tok0, p.ts, p.L, tid);
            walk_gload<false, kThreads>(ro, a.d_o, p.tok0, p.ts, p.L, tid);
        }
        walk_gload<false, kThreads>(rk, a.k, p.tok0, p.ts, p.L, tid);
        walk_gload<false, kThreads>(rw, a.what, p.wtok0, 1, p.L, tid);
    };
    if (cnt > 0) gload(0);

    for (int kk = 0; kk < cnt; ++kk) {
        const ChunkPos cp = walk_pos(d, walk, kend - 1 - kk);
        const int L = cp.L;
        if (MODE != 2) {
            walk_commit<kThreads>(Q, rq, L, tid);
            walk_commit<kThreads>(dO, ro, L, tid);
        }
        walk_commit<kThreads>(K, rk, L, tid);
        walk_commit<kThreads>(Wh, rw, L, tid);
        if (DEC && wave == 0) {
            walk_decay_tables<false>(gval, L, 0.f, bs, wo, lane);
            gm[lane] = __expf(bs[lane]);
        }
        gload(kk + 1);
        __syncthreads();  // (A) tiles and decay tables of this chunk are in LDS
        const float bC = DEC ? bs[C] : 0.f;

        // ---- dS' of this wave's columns -> global, fragment-major: through the wave's private tile [i][v - 32 wave]
        if (MODE == 0) {
        _Pragma("unroll") for (int ib = 0; ib < 4; ++ib)
            _Pragma("unroll") for (int x = 0; x < 16; ++x)
                pw[(32 * ib + 8 * (x >> 2) + 4 * half + (x & 3)) * LDW + n] = uint16_t(pack2(S[ib][x], 0.f));
        __builtin_amdgcn_wave_barrier();
        {
            uint16_t* dst = a.dstates + cp.slot * D * D;
            _Pragma("unroll") for (int blk = 0; blk < 4; ++blk)
                _Pragma("unroll") for (int q2 = 0; q2 < 2; ++q2) {
                    const u32x4 val = *reinterpret_cast<const u32x4*>(pw + (32 * blk + n) * LDW + 16 * q2 + 8 * half);
                    __builtin_nontemporal_store(val, reinterpret_cast<u32x4*>(dst + state_frag_off(blk, 2 * wave + q2, lane)));
                }
        }
        __builtin_amdgcn_wave_barrier();
        }

        // ---- dU^T[v][t] = wo_t sum_i dS'[i][v] k_t[i] + sum_{j >= t} dO[j][v] P[j][t]
        f32x16 dU[2];
        walk_inter<false>(dU, S, K, bs, n, half);
        if (DEC) {
            _Pragma("unroll") for (int tb = 0; tb < 2; ++tb) {
                const float w = wo[32 * tb + n];
                _Pragma("unroll") for (int x = 0; x < 16; ++x) dU[tb][x] *= w;
            }
        }
        if (MODE != 2) {
            walk_scores<DEC>(K, Q, Ph, Pl, bs, wave, n, half);
            __syncthreads();  // (C) scores are in LDS
        }
        _Pragma("unroll") for (int nb = 0; nb < 2; ++nb) {
            if (MODE != 2) {
                _Pragma("unroll") for (int ks = 2 * nb; ks < 4; ++ks) {  // queries j < 32 never see keys t >= 32
                    const bf16x8 dot = frag_tr(dO, LD, 16 * ks, 32 * wave, lane);
                    dU[nb] = mfma(dot, frag_tr(Ph, LDP, 16 * ks, 32 * nb, lane), dU[nb]);
                    dU[nb] = mfma(dot, frag_tr(Pl, LDP, 16 * ks, 32 * nb, lane), dU[nb]);
                }
            }
            const PackedBlock uh = pack_block(dU[nb]);
            f32x16 r = dU[nb];
            _Pragma("unroll") for (int g = 0; g < 4; ++g) {
                r[4 * g + 0] -= bf16_lo(uh.v[g].x);
                r[4 * g + 1] -= bf16_hi(uh.v[g].x);
                r[4 * g + 2] -= bf16_lo(uh.v[g].y);
                r[4 * g + 3] -= bf16_hi(uh.v[g].y);
            }
            store_packed(duh, LDW, 32 * nb + n, 0, half, uh);
            store_packed(dul, LDW, 32 * nb + n, 0, half, pack_block(r));
        }
        __builtin_amdgcn_wave_barrier();
        if (MODE == 0) {
        _Pragma("unroll") for (int it = 0; it < 4; ++it) {
            const int row = (lane >> 2) + 16 * it, piece = lane & 3;
            if (row < L) {
                const size_t off = (cp.wtok0 + row) * D + 32 * wave + 8 * piece;
                *reinterpret_cast<u32x4*>(a.du_h + off) = *reinterpret_cast<const u32x4*>(duh + row * LDW + 8 * piece);
                *reinterpret_cast<u32x4*>(a.du_l + off) = *reinterpret_cast<const u32x4*>(dul + row * LDW + 8 * piece);
            }
        }
        }
        // ---- dS = Gamma_C dS' + sum_t (Gamma_t q_t)^T dO_t - sum_t what_t^T dU_t
        if (DEC) {
            const float lam = __expf(bC);
            _Pragma("unroll") for (int ib = 0; ib < 4; ++ib)
                _Pragma("unroll") for (int x = 0; x < 16; ++x) S[ib][x] *= lam;
        }
        _Pragma("unroll") for (int ks = 0; ks < 4; ++ks) {
            const u32x4 raw = __builtin_bit_cast(u32x4, frag_tr(dO, LD, 16 * ks, 32 * wave, lane));
            u32x4 hi = raw, lo = {0, 0, 0, 0};
            if (DEC) {
                const float4 w0 = *reinterpret_cast<const float4*>(gm + 16 * ks + 8 * half);
                const float4 w1 = *reinterpret_cast<const float4*>(gm + 16 * ks + 8 * half + 4);
                const float w[8] = {w0.x, w0.y, w0.z, w0.w, w1.x, w1.y, w1.z, w1.w};
                _Pragma("unroll") for (int p = 0; p < 4; ++p) {
                    const float x0 = bf16_lo(raw[p]) * w[2 * p], x1 = bf16_hi(raw[p]) * w[2 * p + 1];
                    hi[p] = pack2(x0, x1);
                    lo[p] = pack2(x0 - bf16_lo(hi[p]), x1 - bf16_hi(hi[p]));
                }
            }
            const bf16x8 oh = __builtin_bit_cast(bf16x8, hi), ol = __builtin_bit_cast(bf16x8, lo);
            u32x4 nh = __builtin_bit_cast(u32x4, frag_tr(duh, LDW, 16 * ks, 0, lane));
            u32x4 nl = __builtin_bit_cast(u32x4, frag_tr(dul, LDW, 16 * ks, 0, lane));
            _Pragma("unroll") for (int p = 0; p < 4; ++p) {  // -dU
                nh[p] ^= 0x80008000u;
                nl[p] ^= 0x80008000u;
            }
            const bf16x8 uh = __builtin_bit_cast(bf16x8, nh), ul = __builtin_bit_cast(bf16x8, nl);
            _Pragma("unroll") for (int ib = 0; ib < 4; ++ib) {
                const bf16x8 wa = frag_tr(Wh, LD, 16 * ks, 32 * ib, lane);
                if (MODE != 2) {
                    const bf16x8 qa = frag_tr(Q, LD, 16 * ks, 32 * ib, lane);
                    S[ib] = mfma(qa, oh, S[ib]);
                    if (DEC) S[ib] = mfma(qa, ol, S[ib]);
                }
                S[ib] = mfma(wa, uh, S[ib]);
                S[ib] = mfma(wa, ul, S[ib]);
            }
        }
        __syncthreads();  // (D) every read of this chunk's tiles is done
    }
    if (MODE != 0) {
        walk_state_store(S, a.sum + (size_t(seq) * a.nseg + seg) * D * D, false, wave, n, half);
        return;
    }
    if (a.edge_out && seg == 0) walk_state_store(S, a.edge_out + size_t(seq) * D * D, false, wave, n, half);
}

// ---------------------------------------------------------------------------------------------
// Backward, the chunk-local part: everything that reaches the inputs through the triangular solve.  Per chunk, with
// T = (I + L)^-1, Uhat = T diag(b) V, What = T diag(beta Gamma) K and the gradients dU (of Uhat) and dWhat:
//   dVb = T^T dU          -> dv_r = b_r dVb_r ,            db_r = dVb_r . v_r
//   dKb = T^T dWhat       -> dk_r += beta_r Gamma_r dKb_r , c_r = dKb_r . k_r  (-> d beta_r += Gamma_r c_r, d lg_r += beta_r Gamma_r c_r)
//   dT  = dU (diag(b) V)^T + dWhat (diag(beta Gamma) K)^T   (only its strictly lower part matters)
//   dL  = -T^T dT T^T     (strictly lower part);  L_tr = beta_t e^{lg_t - lg_r} (k_t . k_r):
//   F_tr = dL_tr e^{lg_t - lg_r} (k_t . k_r):  d beta_t += sum_r F_tr ;  d lg_t += beta_t sum_r F_tr ;  d lg_r -= sum_t beta_t F_tr
//   dG_tr = beta_t e^{lg_t - lg_r} dL_tr:      dk_t += sum_r dG_tr k_r ,  dk_r += sum_t dG_tr k_t
// and d log alpha_t = sum_{s >= t} d lg_s inside the chunk (lg is the chunk-local running sum).  The key gradient of
// the gradient walker (head + remainder) is added before the one rounding to bf16, its decay gradient is added to.
struct DeltaGradArgs {
    const uint16_t *k, *v;            // layout of the caller
    const uint16_t *du_h, *du_l, *dw_h, *dw_l;  // [BH*T][128] (library order)
    const uint16_t* tt;               // [BH*N][2][64][64]
    const float *log_alpha, *beta, *bw;
    const uint16_t *dk1_h, *dk1_l;    // the gradient walker's key gradient, layout of the caller
    uint16_t *dk, *dv;
    float *d_log_alpha, *d_beta, *d_bw;   // d_log_alpha is added to
};
// LDS: K | V | dU head | remainder | dWhat head | remainder (64 x LD) | T^T head | remainder | dT head | remainder
// (64 x LDP) | lg, beta, b, e^{lg} | reductions.  After the first phase the five tiles behind K are spent and hold
// M1 = dT T^T and dG (head, remainder, 64 x LDP each) and the stages of dv and dk.
constexpr int kDeltaGradRed = (4 * C + 4 * 2 * C + 3 * C + 3 * C) * 4;  // params | db, c per wave | row sums | column sums
constexpr int kDeltaGradLds = 6 * C * LD * 2 + 4 * C * LDP * 2 + kDeltaGradRed;

// grid: up to one workgroup per compute unit; each takes chunks blockIdx.x, blockIdx.x + gridDim.x, ...
template <bool DEC>
__global__ __launch_bounds__(kThreads, 1) void mk_delta_grad(Dims d, DeltaGradArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    uint16_t* K = reinterpret_cast<uint16_t*>(smem);
    uint16_t* V = K + C * LD;
    uint16_t* dUh = V + C * LD;
    uint16_t* dUl = dUh + C * LD;
    uint16_t* dWh = dUl + C * LD;
    uint16_t* dWl = dWh + C * LD;
    uint16_t* TTh = dWl + C * LD;
    uint16_t* TTl = TTh + C * LDP;
    uint16_t* dTh = TTl + C * LDP;
    uint16_t* dTl = dTh + C * LDP;
    float* lg = reinterpret_cast<float*>(dTl + C * LDP);
    float* be = lg + C;
    float* bb = be + C;
    float* gm = bb + C;           // e^{lg}
    float* red_db = gm + C;       // [wave][64]
    float* red_c = red_db + 4 * C;
    float* rowF = red_c + 4 * C;  // [3 blocks][32]: sum_r F_tr per t of the block
    float* colE = rowF + 3 * C;   // [3 blocks][32]: sum_t beta_t F_tr per r of the block   (3 * C floats reserved each)
    // second phase, over V .. dWl
    uint16_t* M1h = V;
    uint16_t* M1l = M1h + C * LDP;
    uint16_t* dGh = M1l + C * LDP;
    uint16_t* dGl = dGh + C * LDP;
    uint16_t* stv = dGl + C * LDP;   // stage of dv (64 x LD)
    uint16_t* stk = stv + C * LD;    // stage of dk
    static_assert(4 * C * LDP + 2 * C * LD <= 5 * C * LD, "second phase fits behind K");

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), n = lane & 31, half = lane >> 5;
    const int jobs = d.N * d.BH();
    // One workgroup per compute unit walks over chunks; the rows of the next chunk are requested into registers while
    // this one is worked on (the kernel needs most of the unit's LDS, so no second workgroup hides the loads).
    struct Pre { TileRegs k, v, uh, ul, wh, wl; u32x4 tt[4]; float la, be, bw; } pre;
    auto gload = [&](int job) {
        const ChunkPos p = chunk_pos(d, job % d.N, job / d.N);
        const int Lp = max(p.L, 1);
        const size_t pt = p.tok0 + size_t(min(lane, Lp - 1)) * p.ts;
        pre.la = DEC ? a.log_alpha[pt] : 0.f;
        pre.be = a.beta ? a.beta[pt] : 1.f;
        pre.bw = a.bw ? a.bw[pt] : 1.f;
        tile_gload(pre.k, a.k, p.tok0, p.ts, Lp, tid);
        tile_gload(pre.v, a.v, p.tok0, p.ts, Lp, tid);
        tile_gload(pre.uh, a.du_h, p.wtok0, 1, Lp, tid);
        tile_gload(pre.ul, a.du_l, p.wtok0, 1, Lp, tid);
        tile_gload(pre.wh, a.dw_h, p.wtok0, 1, Lp, tid);
        tile_gload(pre.wl, a.dw_l, p.wtok0, 1, Lp, tid);
        const uint16_t* gtt = a.tt + p.slot * 2 * C * C;
        _Pragma("unroll") for (int it = 0; it < 4; ++it) {
            const int q = tid + kThreads * it, plane = q >> 9, row = (q >> 3) & 63, piece = q & 7;
            pre.tt[it] = *reinterpret_cast<const u32x4*>(gtt + plane * C * C + row * C + 8 * piece);
        }
    };
    if (int(blockIdx.x) < jobs) gload(blockIdx.x);
  for (int job = blockIdx.x; job < jobs; job += gridDim.x) {
    const ChunkPos cp = chunk_pos(d, job % d.N, job / d.N);
    const int L = cp.L;
    const size_t ptok = cp.tok0 + size_t(min(lane, max(L, 1) - 1)) * cp.ts;
    if (wave == 0) {
        float x = (DEC && lane < L) ? pre.la : 0.f;
        for (int off = 1; off < 64; off <<= 1) {
            const float y = __shfl_up(x, off, 64);
            if (lane >= off) x += y;
        }
        lg[lane] = x;
        be[lane] = lane < L ? pre.be : 0.f;
        bb[lane] = lane < L ? pre.bw : 0.f;
        gm[lane] = DEC ? __expf(x) : 1.f;
    }
    tile_commit(K, pre.k, L, tid);
    tile_commit(V, pre.v, L, tid);
    tile_commit(dUh, pre.uh, L, tid);
    tile_commit(dUl, pre.ul, L, tid);
    tile_commit(dWh, pre.wh, L, tid);
    tile_commit(dWl, pre.wl, L, tid);
    _Pragma("unroll") for (int it = 0; it < 4; ++it) {
        const int q = tid + kThreads * it, plane = q >> 9, row = (q >> 3) & 63, piece = q & 7;
        *reinterpret_cast<u32x4*>((plane ? TTl : TTh) + row * LDP + 8 * piece) = pre.tt[it];
    }
    // the gradient walker's key gradient of this chunk (both planes), wanted at the very end
    u32x2 k1h[2][4], k1l[2][4];
    _Pragma("unroll") for (int nb = 0; nb < 2; ++nb) {
        const size_t row = (cp.tok0 + size_t(min(32 * nb + n, max(L, 1) - 1)) * cp.ts) * D + 32 * wave + 4 * half;
        _Pragma("unroll") for (int g = 0; g < 4; ++g) {
            k1h[nb][g] = *reinterpret_cast<const u32x2*>(a.dk1_h + row + 8 * g);
            k1l[nb][g] = *reinterpret_cast<const u32x2*>(a.dk1_l + row + 8 * g);
        }
    }
    if (job + int(gridDim.x) < jobs) gload(job + gridDim.x);
    __syncthreads();

    // ---- first phase
    PackedBlock resv[2];
    f32x16 dk2[2];
    _Pragma("unroll") for (int nb = 0; nb < 2; ++nb) {
        // dVb^T[v][r] = sum_t dU[t][v] T[t][r],  dKb^T[i][r] = sum_t dWhat[t][i] T[t][r]  (T[t][r] = 0 for t < r)
        f32x16 av = {0}, ak = {0};
        _Pragma("unroll") for (int ks = 2 * nb; ks < 4; ++ks) {
            const bf16x8 th = frag(TTh, LDP, 32 * nb + n, 16 * ks + 8 * half), tl = frag(TTl, LDP, 32 * nb + n, 16 * ks + 8 * half);
            const bf16x8 uh = frag_tr(dUh, LD, 16 * ks, 32 * wave, lane), ul = frag_tr(dUl, LD, 16 * ks, 32 * wave, lane);
            const bf16x8 wh = frag_tr(dWh, LD, 16 * ks, 32 * wave, lane), wl = frag_tr(dWl, LD, 16 * ks, 32 * wave, lane);
            av = mfma(uh, th, av);
            av = mfma(uh, tl, av);
            av = mfma(ul, th, av);
            ak = mfma(wh, th, ak);
            ak = mfma(wh, tl, ak);
            ak = mfma(wl, th, ak);
        }
        const int r = 32 * nb + n;
        float pdb = row_dot(V, r, wave, half, av), pc = row_dot(K, r, wave, half, ak);
        pdb += __shfl_xor(pdb, 32, 64);
        pc += __shfl_xor(pc, 32, 64);
        if (half == 0) {
            red_db[wave * C + r] = pdb;
            red_c[wave * C + r] = pc;
        }
        const float br = bb[r], wr = be[r] * gm[r];
        _Pragma("unroll") for (int x = 0; x < 16; ++x) {
            av[x] *= br;
            ak[x] *= wr;
        }
        resv[nb] = pack_block(av);
        dk2[nb] = ak;
    }
    // dT[t][r] for r < t, blocks (r, t) = (0,0), (0,1), (1,1) by waves 0, 1, 2; wave 3 clears the block above the diagonal
    if (wave < 3) {
        const int rb = wave == 2 ? 1 : 0, tb = wave ? 1 : 0;
        f32x16 t1 = score_block2(V, 32 * rb, dUh, 32 * tb, n, half);   // D[m = r][n = t] = v_r . dU_t
        t1 = score_block2(V, 32 * rb, dUl, 32 * tb, n, half, t1);
        f32x16 t2 = score_block2(K, 32 * rb, dWh, 32 * tb, n, half);
        t2 = score_block2(K, 32 * rb, dWl, 32 * tb, n, half, t2);
        const int t = 32 * tb + n;
        _Pragma("unroll") for (int g = 0; g < 4; ++g) {
            const int r0 = 32 * rb + 8 * g + 4 * half;
            const float4 b4 = *reinterpret_cast<const float4*>(bb + r0), e4 = *reinterpret_cast<const float4*>(be + r0);
            const float4 g4 = *reinterpret_cast<const float4*>(gm + r0);
            const float bv[4] = {b4.x, b4.y, b4.z, b4.w}, wv[4] = {e4.x * g4.x, e4.y * g4.y, e4.z * g4.z, e4.w * g4.w};
            _Pragma("unroll") for (int j = 0; j < 4; ++j)
                t1[4 * g + j] = (r0 + j < t) ? t1[4 * g + j] * bv[j] + t2[4 * g + j] * wv[j] : 0.f;
        }
        store_block_t_split(dTh, dTl, LDP, t, 32 * rb, half, t1);
    } else {
        _Pragma("unroll") for (int it = 0; it < 2; ++it) {   // rows t < 32, columns r >= 32
            const int p = lane + 64 * it, row = p >> 2, piece = p & 3;
            *reinterpret_cast<u32x4*>(dTh + row * LDP + 32 + 8 * piece) = u32x4{0, 0, 0, 0};
            *reinterpret_cast<u32x4*>(dTl + row * LDP + 32 + 8 * piece) = u32x4{0, 0, 0, 0};
        }
    }
    __syncthreads();  // first phase done: the tiles behind K are spent, dT is complete

    // ---- M1[t][r] = sum_r' dT[t][r'] T[r][r'], blocks (r, t) = (0,0), (0,1), (1,1); kept as a tile [t][r]
    if (wave < 3) {
        const int mb = wave == 2 ? 1 : 0, nb = wave ? 1 : 0;
        f32x16 m1 = {0};
        _Pragma("unroll") for (int ks = 0; ks < 4; ++ks) {
            if (ks >= 2 * (mb + 1)) break;  // r' <= r
            const bf16x8 ah = frag_tr(TTh, LDP, 16 * ks, 32 * mb, lane), al = frag_tr(TTl, LDP, 16 * ks, 32 * mb, lane);  // T[r][r']
            const bf16x8 bh_ = frag(dTh, LDP, 32 * nb + n, 16 * ks + 8 * half), bl = frag(dTl, LDP, 32 * nb + n, 16 * ks + 8 * half);
            m1 = mfma(ah, bh_, m1);
            m1 = mfma(ah, bl, m1);
            m1 = mfma(al, bh_, m1);
        }
        store_block_t_split(M1h, M1l, LDP, 32 * nb + n, 32 * mb, half, m1);
    } else {
        _Pragma("unroll") for (int it = 0; it < 2; ++it) {   // rows t' < 32, columns r >= 32: never contribute
            const int p = lane + 64 * it, row = p >> 2, piece = p & 3;
            *reinterpret_cast<u32x4*>(M1h + row * LDP + 32 + 8 * piece) = u32x4{0, 0, 0, 0};
            *reinterpret_cast<u32x4*>(M1l + row * LDP + 32 + 8 * piece) = u32x4{0, 0, 0, 0};
            *reinterpret_cast<u32x4*>(dGh + row * LDP + 32 + 8 * piece) = u32x4{0, 0, 0, 0};
            *reinterpret_cast<u32x4*>(dGl + row * LDP + 32 + 8 * piece) = u32x4{0, 0, 0, 0};
        }
    }
    __syncthreads();
    // ---- dL[t][r] = -sum_t' T[t'][t] M1[t'][r], then F, the row and column sums, and dG as a tile [t][r]
    if (wave < 3) {
        const int mb = wave == 2 ? 1 : 0, nb = wave ? 1 : 0;
        f32x16 dl = {0};
        _Pragma("unroll") for (int ks = 2 * nb; ks < 4; ++ks) {  // t' >= t
            const bf16x8 ah = frag_tr(M1h, LDP, 16 * ks, 32 * mb, lane), al = frag_tr(M1l, LDP, 16 * ks, 32 * mb, lane);  // M1[t'][r]
            const bf16x8 bh_ = frag(TTh, LDP, 32 * nb + n, 16 * ks + 8 * half), bl = frag(TTl, LDP, 32 * nb + n, 16 * ks + 8 * half);  // T[t'][t]
            dl = mfma(ah, bh_, dl);
            dl = mfma(ah, bl, dl);
            dl = mfma(al, bh_, dl);
        }
        const f32x16 G = score_block2(K, 32 * mb, K, 32 * nb, n, half);  // D[m = r][n = t] = k_r . k_t
        const int t = 32 * nb + n;
        const float bt = be[t], lt = lg[t];
        float rs = 0.f;
        f32x16 dg;
        float cs[16];
        _Pragma("unroll") for (int g = 0; g < 4; ++g) {
            const int r0 = 32 * mb + 8 * g + 4 * half;
            const float4 l4 = *reinterpret_cast<const float4*>(lg + r0);
            const float lr[4] = {l4.x, l4.y, l4.z, l4.w};
            _Pragma("unroll") for (int j = 0; j < 4; ++j) {
                const float dec = DEC ? __expf(lt - lr[j]) : 1.f;
                const float dlv = (r0 + j < t) ? -dl[4 * g + j] * dec : 0.f;   // dL_tr e^{lg_t - lg_r}
                const float f = dlv * G[4 * g + j];
                rs += f;
                cs[4 * g + j] = bt * f;
                dg[4 * g + j] = bt * dlv;
            }
        }
        rs += __shfl_xor(rs, 32, 64);
        if (half == 0) rowF[wave * 32 + n] = rs;
        if (DEC) {  // column sums over the 32 tokens t of the block, for each r
            _Pragma("unroll") for (int x = 0; x < 16; ++x) {
                float v_ = cs[x];
                for (int off = 16; off > 0; off >>= 1) v_ += __shfl_xor(v_, off, 64);
                cs[x] = v_;
            }
            if (n == 0) {
                _Pragma("unroll") for (int x = 0; x < 16; ++x) colE[wave * 32 + 8 * (x >> 2) + 4 * half + (x & 3)] = cs[x];
            }
        }
        store_block_t_split(dGh, dGl, LDP, t, 32 * mb, half, dg);
    }
    __syncthreads();
    // ---- dk^T[i][t] = dk2[i][t] + sum_r K^T[i][r] (dG[t][r] + dG[r][t]) + the gradient walker's part
    _Pragma("unroll") for (int nb = 0; nb < 2; ++nb) {
        f32x16 acc = dk2[nb];
        _Pragma("unroll") for (int ks = 0; ks < 4; ++ks) {
            const bf16x8 kt = frag_tr(K, LD, 16 * ks, 32 * wave, lane);
            if (ks < 2 * (nb + 1)) {  // r < t
                acc = mfma(kt, frag(dGh, LDP, 32 * nb + n, 16 * ks + 8 * half), acc);
                acc = mfma(kt, frag(dGl, LDP, 32 * nb + n, 16 * ks + 8 * half), acc);
            }
            if (ks >= 2 * nb) {       // r > t
                acc = mfma(kt, frag_tr(dGh, LDP, 16 * ks, 32 * nb, lane), acc);
                acc = mfma(kt, frag_tr(dGl, LDP, 16 * ks, 32 * nb, lane), acc);
            }
        }
        const int t = 32 * nb + n;
        _Pragma("unroll") for (int g = 0; g < 4; ++g) {
            const u32x2 h = k1h[nb][g], l = k1l[nb][g];
            acc[4 * g + 0] += bf16_lo(h.x) + bf16_lo(l.x);
            acc[4 * g + 1] += bf16_hi(h.x) + bf16_hi(l.x);
            acc[4 * g + 2] += bf16_lo(h.y) + bf16_lo(l.y);
            acc[4 * g + 3] += bf16_hi(h.y) + bf16_hi(l.y);
        }
        store_packed(stk, LD, t, 32 * wave, half, pack_block(acc));
        store_packed(stv, LD, t, 32 * wave, half, resv[nb]);
    }
    __syncthreads();
    store_tile(a.dk, stk, cp.tok0, cp.ts, L, tid);
    store_tile(a.dv, stv, cp.tok0, cp.ts, L, tid);
    // ---- per-token parameters (wave 0, lane = token)
    if (wave == 0) {
        const int t = lane;
        const float cb = (red_c[t] + red_c[C + t]) + (red_c[2 * C + t] + red_c[3 * C + t]);
        const float db = (red_db[t] + red_db[C + t]) + (red_db[2 * C + t] + red_db[3 * C + t]);
        // row sums of F: t < 32 from block 0; t >= 32 from blocks 1 and 2.  Column sums: r < 32 from blocks 0 and 1; r >= 32 from block 2.
        const float rf = t < 32 ? rowF[t] : rowF[32 + (t - 32)] + rowF[64 + (t - 32)];
        if (a.d_bw && t < L) a.d_bw[ptok] = db;
        if (a.d_beta && t < L) a.d_beta[ptok] = gm[t] * cb + rf;
        if (DEC) {
            const float ce = t < 32 ? colE[t] + colE[32 + t] : colE[64 + (t - 32)];
            float dlg = be[t] * gm[t] * cb + be[t] * rf - ce;
            if (t >= L) dlg = 0.f;
            float sfx = dlg;  // suffix sum over tokens >= t
            for (int off = 1; off < 64; off <<= 1) {
                const float y = __shfl_down(sfx, off, 64);
                if (t + off < 64) sfx += y;
            }
            if (t < L) a.d_log_alpha[ptok] += sfx;
        }
    }
    __syncthreads();  // the stages and the reductions are read; the next chunk may overwrite them
  }
}
