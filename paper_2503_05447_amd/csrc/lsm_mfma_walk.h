// Fused chunk walkers of the scalar decay kinds (none / per head / per token): bf16 operands, fp32
// accumulation, chunk = 64, d_k = d_v = 128.  Included by lsm_mfma.hip.
//
// One workgroup walks a run of consecutive chunks (a "segment") of one (b,h) recurrence with the
// 128 x 128 state in MFMA accumulators, so the forward pass writes no per-chunk state at all and the
// backward pass only the state gradients.  Per chunk the forward walker evaluates Algorithm 2 of the
// paper with the decay folded in,
//     o_t = e^{b_t} q_t S + sum_{r <= t} (q_t . k_r) e^{b_t - b_r} v_r        (O_inter + O_intra)
//     S  <- e^{b_C} S + sum_r e^{b_C - b_r} k_r^T v_r                         (chunk state, prefix)
// and the gradient walker (further down) the adjoint of the same chunk with S carried the same way.
//
// Segments: with fewer recurrences than the chip can keep busy a sequence is cut into segments of m
// chunks.  A first pass (SUMMARY: the state update alone, from a zero state) leaves each segment's own
// contribution and total log-decay, a small scan turns them into the state every segment starts from,
// and the walkers then run all segments in parallel.  Only those entry states (one per m chunks) ever
// reach memory.  REV walks backward in time (a chunk's rows are loaded in reverse token order and beta
// is the exclusive instead of the inclusive running sum of the log-decays in walk order); it serves
// the summary pass of the reverse direction.
#pragma once

struct WalkArgs {
    const uint16_t *xq, *xk, *xv;  // rows in the query, key and value role (forward pass: q, k, v)
    const float* g;                // log-decay (per kind)
    uint16_t* out;
    const float* edge_in;  // state a whole sequence starts from, [i][v] fp32 per sequence; NULL = zero
    float* edge_out;       // state it ends with; NULL = not wanted
    float* bound;          // [seqs][nseg][128 x 128] fp32, [i][v]: entry state of every segment (nseg > 1)
    float* gseg;           // [seqs][nseg]: total log-decay of each segment (SUMMARY writes)
    int m, nseg;           // chunks per segment, segments per sequence (upper bound for packed input)
    int skip;              // SUMMARY, REV: segments [0, skip) feed no other walk and are left out (at least 1)
    const uint16_t* xv_lo; // VSPLIT (summary pass only): remainder plane of the value-role rows
};

// tile rows in walk order: row r holds token r (forward) or token L-1-r (backward); rows >= L are zero.
// NT threads share a tile: 1024 / NT pieces of 16 bytes each.
template <bool REV, int NT>
__device__ __forceinline__ void walk_gload(TileRegs& r, const uint16_t* src, size_t tok0, int ts, int L, int tid) {
    // uniform base (scalar registers) + a 32-bit byte offset per lane, shared by every tile of the chunk
    const char* base = reinterpret_cast<const char*>(src + tok0 * D);
    _Pragma("unroll") for (int it = 0; it < 1024 / NT; ++it) {
        const int p = tid + NT * it, row = min(p >> 4, L - 1), cp = p & 15;
        const int tok = REV ? L - 1 - row : row;
        const uint32_t off = (uint32_t(tok) * uint32_t(ts) * D + cp * 8) * 2;
        r.v[it] = *reinterpret_cast<const u32x4*>(base + off);
    }
}
template <int NT>
__device__ __forceinline__ void walk_commit(uint16_t* dst, const TileRegs& r, int L, int tid) {
    _Pragma("unroll") for (int it = 0; it < 1024 / NT; ++it) {
        const int p = tid + NT * it, row = p >> 4, cp = p & 15;
        const uint32_t keep = row < L ? 0xffffffffu : 0u;
        *reinterpret_cast<u32x4*>(dst + row * LD + cp * 8) = u32x4{r.v[it].x & keep, r.v[it].y & keep, r.v[it].z & keep, r.v[it].w & keep};
    }
}
// NT threads store an output stage
template <bool REV, int NT = kThreads>
__device__ __forceinline__ void walk_store(uint16_t* dst, const uint16_t* src, size_t tok0, int ts, int L, int tid) {
    char* base = reinterpret_cast<char*>(dst + tok0 * D);
    _Pragma("unroll") for (int it = 0; it < 1024 / NT; ++it) {
        const int p = tid + NT * it, row = p >> 4, cp = p & 15;
        const uint32_t off = (uint32_t(REV ? L - 1 - row : row) * uint32_t(ts) * D + cp * 8) * 2;
        if (row < L)
            __builtin_nontemporal_store(*reinterpret_cast<const u32x4*>(src + row * LD + cp * 8), reinterpret_cast<u32x4*>(base + off));
    }
}

// B operand whose k order follows a D-layout block used as A operand: slot e of lane (n, half) is
// column col0 + 8 (e / 4) + 4 half + e % 4 of row `row`
__device__ __forceinline__ bf16x8 frag_perm(const uint16_t* tile, int ld, int row, int col0, int half) {
    const u32x2 a = *reinterpret_cast<const u32x2*>(tile + row * ld + col0 + 4 * half);
    const u32x2 b = *reinterpret_cast<const u32x2*>(tile + row * ld + col0 + 8 + 4 * half);
    return __builtin_bit_cast(bf16x8, u32x4{a.x, a.y, b.x, b.y});
}

// mask (key r <= query j) and decay e^{beta_j - beta_r} of a score block whose rows index keys
template <bool DEC>
__device__ __forceinline__ void walk_mask(f32x16& acc, int m0, int ncol, const float* bs, int half) {
    const float bn = DEC ? bs[ncol] : 0.f;
    _Pragma("unroll") for (int g = 0; g < 4; ++g) {
        float bmv[4] = {0.f, 0.f, 0.f, 0.f};
        if (DEC) {
            const float4 bm = *reinterpret_cast<const float4*>(bs + m0 + 8 * g + 4 * half);
            bmv[0] = bm.x; bmv[1] = bm.y; bmv[2] = bm.z; bmv[3] = bm.w;
        }
        _Pragma("unroll") for (int jj = 0; jj < 4; ++jj) {
            const int r = m0 + 8 * g + 4 * half + jj, x = 4 * g + jj;
            const float w = DEC ? __expf(bn - bmv[jj]) : 1.f;
            acc[x] = r <= ncol ? acc[x] * w : 0.f;
        }
    }
}

__host__ __device__ constexpr int walk_lds(bool summary) {
    return summary ? 2 * C * LD * 2 + (2 * C + 8) * 4 : (3 * C * LD + 2 * C * LDP) * 2 + (2 * C + 8) * 4;
}

// D[m][n] = sum_f Am[m0 + m][f] * Bm[n0 + n][f] over the 128 features of two row-major LDS tiles, the
// fragments requested four k-steps at a time (a lower register peak than all sixteen at once)
__device__ __forceinline__ f32x16 score_block2(const uint16_t* Am, int m0, const uint16_t* Bm, int n0, int n, int half,
                                               f32x16 acc = f32x16{0}) {
    _Pragma("unroll") for (int h4 = 0; h4 < 2; ++h4) {
        bf16x8 fa[4], fb[4];
        _Pragma("unroll") for (int ks = 0; ks < 4; ++ks) {
            fa[ks] = frag(Am, LD, m0 + n, 16 * (4 * h4 + ks) + 8 * half);
            fb[ks] = frag(Bm, LD, n0 + n, 16 * (4 * h4 + ks) + 8 * half);
        }
        _Pragma("unroll") for (int ks = 0; ks < 4; ++ks) acc = mfma(fa[ks], fb[ks], acc);
    }
    return acc;
}

// ---- the four contractions of one chunk for the wave that owns value features [32 w4, 32 w4 + 32)
// state block ib: S[ib][4g+j] = state[key feature 32 ib + 8g + 4 half + j][value feature 32 w4 + n]

// inter: O^T[v][j] = e^{beta_j} sum_i S[i][v] q_j[i], the state blocks as A operands straight from the
// accumulators (bf16 head + remainder), the query rows read in the matching k order
template <bool DEC>
__device__ __forceinline__ void walk_inter(f32x16 (&O)[2], const f32x16 (&S)[4], const uint16_t* Q, const float* bs, int n, int half) {
    O[0] = f32x16{0};
    O[1] = f32x16{0};
    _Pragma("unroll") for (int ib = 0; ib < 4; ++ib)
        _Pragma("unroll") for (int p = 0; p < 2; ++p) {
            u32x4 hi, lo;
            _Pragma("unroll") for (int e = 0; e < 4; ++e) {
                const float x0 = S[ib][8 * p + 2 * e], x1 = S[ib][8 * p + 2 * e + 1];
                hi[e] = pack2(x0, x1);
                lo[e] = pack2(x0 - bf16_lo(hi[e]), x1 - bf16_hi(hi[e]));
            }
            const bf16x8 sh = __builtin_bit_cast(bf16x8, hi), sl = __builtin_bit_cast(bf16x8, lo);
            const bf16x8 qf0 = frag_perm(Q, LD, n, 32 * ib + 16 * p, half);
            const bf16x8 qf1 = frag_perm(Q, LD, 32 + n, 32 * ib + 16 * p, half);
            O[0] = mfma(sh, qf0, O[0]);
            O[1] = mfma(sh, qf1, O[1]);
            O[0] = mfma(sl, qf0, O[0]);
            O[1] = mfma(sl, qf1, O[1]);
        }
    if (DEC) {
        _Pragma("unroll") for (int jb = 0; jb < 2; ++jb) {
            const float w = __expf(bs[32 * jb + n]);
            _Pragma("unroll") for (int x = 0; x < 16; ++x) O[jb][x] *= w;
        }
    }
}
// two inter products against the same state with one conversion of its blocks: Oa^T = S^T A^T (unscaled), Ob^T = e^{beta} S^T B^T
template <bool DEC, bool WANT_B>
__device__ __forceinline__ void walk_inter_pair(f32x16 (&Oa)[2], f32x16 (&Ob)[2], const f32x16 (&S)[4], const uint16_t* A, const uint16_t* B,
                                                const float* bs, int n, int half) {
    _Pragma("unroll") for (int jb = 0; jb < 2; ++jb) {
        Oa[jb] = f32x16{0};
        Ob[jb] = f32x16{0};
    }
    _Pragma("unroll") for (int ib = 0; ib < 4; ++ib)
        _Pragma("unroll") for (int p = 0; p < 2; ++p) {
            u32x4 hi, lo;
            _Pragma("unroll") for (int e = 0; e < 4; ++e) {
                const float x0 = S[ib][8 * p + 2 * e], x1 = S[ib][8 * p + 2 * e + 1];
                hi[e] = pack2(x0, x1);
                lo[e] = pack2(x0 - bf16_lo(hi[e]), x1 - bf16_hi(hi[e]));
            }
            const bf16x8 sh = __builtin_bit_cast(bf16x8, hi), sl = __builtin_bit_cast(bf16x8, lo);
            const bf16x8 a0 = frag_perm(A, LD, n, 32 * ib + 16 * p, half), a1 = frag_perm(A, LD, 32 + n, 32 * ib + 16 * p, half);
            Oa[0] = mfma(sh, a0, Oa[0]);
            Oa[1] = mfma(sh, a1, Oa[1]);
            Oa[0] = mfma(sl, a0, Oa[0]);
            Oa[1] = mfma(sl, a1, Oa[1]);
            if (WANT_B) {
                const bf16x8 b0 = frag_perm(B, LD, n, 32 * ib + 16 * p, half), b1 = frag_perm(B, LD, 32 + n, 32 * ib + 16 * p, half);
                Ob[0] = mfma(sh, b0, Ob[0]);
                Ob[1] = mfma(sh, b1, Ob[1]);
                Ob[0] = mfma(sl, b0, Ob[0]);
                Ob[1] = mfma(sl, b1, Ob[1]);
            }
        }
    if (DEC && WANT_B) {
        _Pragma("unroll") for (int jb = 0; jb < 2; ++jb) {
            const float w = __expf(bs[32 * jb + n]);
            _Pragma("unroll") for (int x = 0; x < 16; ++x) Ob[jb][x] *= w;
        }
    }
}
// scores: each of the three 32 x 32 blocks on or below the diagonal by one wave (w4 = 0: (0,0), 1: (1,0),
// 2: (1,1)), mask and decay on its accumulators, handed to the others through LDS as head + remainder
template <bool DEC>
__device__ __forceinline__ void walk_scores(const uint16_t* K, const uint16_t* Q, uint16_t* Ph, uint16_t* Pl, const float* bs,
                                            int w4, int n, int half) {
    if (w4 >= 3) return;
    const int pjb = w4 ? 1 : 0, prb = w4 == 2 ? 1 : 0;
    f32x16 P = score_block2(K, 32 * prb, Q, 32 * pjb, n, half);  // D[m = r][n = j] = k_r . q_j
    walk_mask<DEC>(P, 32 * prb, 32 * pjb + n, bs, half);
    store_block_t_split(Ph, Pl, LDP, 32 * pjb + n, 32 * prb, half, P);
}
// intra: O^T[v][j] += sum_{r <= j} V^T[v][r] P[j][r] for the query block jb
__device__ __forceinline__ void walk_intra(f32x16& O, int jb, const uint16_t* V, const uint16_t* Ph, const uint16_t* Pl, int w4,
                                           int lane, int n, int half) {
    const int j = 32 * jb + n;
    _Pragma("unroll") for (int ks = 0; ks < 4; ++ks) {
        if (ks >= 2 * (jb + 1)) break;  // keys r >= 32 never reach queries j < 32
        const bf16x8 vt = frag_tr(V, LD, 16 * ks, 32 * w4, lane);
        O = mfma(vt, frag(Ph, LDP, j, 16 * ks + 8 * half), O);
        O = mfma(vt, frag(Pl, LDP, j, 16 * ks + 8 * half), O);
    }
}
// state: S[i][v] = e^{b_C} S[i][v] + sum_t K^T[i][t] (wo_t V[t][v]); the weighted value slice of this wave is
// split into head + remainder in registers.  SCALE = false: the weights already carry every decay.
// K2 (KSPLIT): remainder plane of the key-role tile (remainder x remainder is left out).
template <bool DEC, bool SCALE, bool KSPLIT = false>
__device__ __forceinline__ void walk_update(f32x16 (&S)[4], const uint16_t* K, const uint16_t* V, const float* wo, float bC, int w4,
                                            int lane, int half, const uint16_t* K2 = nullptr) {
    if (DEC && SCALE) {
        const float lam = __expf(bC);
        _Pragma("unroll") for (int ib = 0; ib < 4; ++ib)
            _Pragma("unroll") for (int x = 0; x < 16; ++x) S[ib][x] *= lam;
    }
    _Pragma("unroll") for (int ks = 0; ks < 4; ++ks) {
        const u32x4 raw = __builtin_bit_cast(u32x4, frag_tr(V, LD, 16 * ks, 32 * w4, lane));
        u32x4 hi = raw, lo = {0, 0, 0, 0};
        if (DEC) {
            const float4 w0 = *reinterpret_cast<const float4*>(wo + 16 * ks + 8 * half);
            const float4 w1 = *reinterpret_cast<const float4*>(wo + 16 * ks + 8 * half + 4);
            const float w[8] = {w0.x, w0.y, w0.z, w0.w, w1.x, w1.y, w1.z, w1.w};
            _Pragma("unroll") for (int p = 0; p < 4; ++p) {
                const float x0 = bf16_lo(raw[p]) * w[2 * p], x1 = bf16_hi(raw[p]) * w[2 * p + 1];
                hi[p] = pack2(x0, x1);
                lo[p] = pack2(x0 - bf16_lo(hi[p]), x1 - bf16_hi(hi[p]));
            }
        }
        const bf16x8 vh = __builtin_bit_cast(bf16x8, hi), vl = __builtin_bit_cast(bf16x8, lo);
        bf16x8 ka[4];
        _Pragma("unroll") for (int ib = 0; ib < 4; ++ib) ka[ib] = frag_tr(K, LD, 16 * ks, 32 * ib, lane);
        _Pragma("unroll") for (int ib = 0; ib < 4; ++ib) S[ib] = mfma(ka[ib], vh, S[ib]);
        if (DEC) {
            _Pragma("unroll") for (int ib = 0; ib < 4; ++ib) S[ib] = mfma(ka[ib], vl, S[ib]);
        }
        if (KSPLIT) {
            _Pragma("unroll") for (int ib = 0; ib < 4; ++ib) S[ib] = mfma(frag_tr(K2, LD, 16 * ks, 32 * ib, lane), vh, S[ib]);
        }
    }
}
// the same state update with the values in two planes (head + remainder; the pseudo-values of the delta rule), the
// weighted slice split again into head + remainder in registers
template <bool DEC, bool SCALE>
__device__ __forceinline__ void walk_update_vsplit(f32x16 (&S)[4], const uint16_t* K, const uint16_t* Vh, const uint16_t* Vl,
                                             const float* wo, float bC, int w4, int lane, int half) {
    if (DEC && SCALE) {
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

// chunk-local decay tables by one wave: beta (inclusive running sum of the log-decays in walk order, exclusive
// when walking backward), b_C, and the weights wo = e^{b_C - beta + extra} of the state update
template <bool REV>
__device__ __forceinline__ float walk_decay_tables(float gval, int L, float extra, float* bs, float* wo, int lane) {
    const float x = lane < L ? gval : 0.f;
    float inc = x;
    for (int off = 1; off < 64; off <<= 1) {
        const float y = __shfl_up(inc, off, 64);
        if (lane >= off) inc += y;
    }
    const float bC = __shfl(inc, 63, 64), beta = REV ? inc - x : inc;
    bs[lane] = beta;
    wo[lane] = __expf(bC - beta + extra);
    if (lane == 0) bs[C] = bC;
    return bC;
}
// state block layout <-> the [i][v] fp32 arrays (transposed: the walker's state is the transpose of the array)
// (erow: row stride of the array; the caller's states have d_v columns, the library's own 128)
__device__ __forceinline__ void walk_state_load(f32x16 (&S)[4], const float* e, bool transposed, int w4, int n, int half, int erow = D) {
    _Pragma("unroll") for (int ib = 0; ib < 4; ++ib)
        _Pragma("unroll") for (int x = 0; x < 16; ++x) {
            const int mm = 32 * ib + 8 * (x >> 2) + 4 * half + (x & 3), nn = 32 * w4 + n;
            S[ib][x] = transposed ? e[nn * erow + mm] : e[mm * erow + nn];
        }
}
__device__ __forceinline__ void walk_state_store(const f32x16 (&S)[4], float* e, bool transposed, int w4, int n, int half, int erow = D) {
    _Pragma("unroll") for (int ib = 0; ib < 4; ++ib)
        _Pragma("unroll") for (int x = 0; x < 16; ++x) {
            const int mm = 32 * ib + 8 * (x >> 2) + 4 * half + (x & 3), nn = 32 * w4 + n;
            e[transposed ? nn * erow + mm : mm * erow + nn] = S[ib][x];
        }
}
// the caller's state of recurrence `seq` ([d_k][d_v] fp32), at the value slice of this pass
__device__ __forceinline__ size_t edge_off(const Dims& d, int seq) { return (size_t(seq) * D * d.vm + d.vs) * D; }
// REV: walk backward in time.  DEC: a decay is present.  SUMMARY: the state update alone, from a zero
// state, result to a.bound / a.gseg.
template <bool REV, bool DEC, bool SUMMARY, bool VSPLIT = false>
__device__ __forceinline__ void walk_body(const Dims& d, const WalkArgs& a, int seq, int seg, unsigned char* smem) {
    // LDS: SUMMARY: K | V | bs | wo;   else: Q | K | V | P head | P remainder | bs | wo
    uint16_t* Q = reinterpret_cast<uint16_t*>(smem);
    uint16_t* K = SUMMARY ? Q : Q + C * LD;
    uint16_t* V = K + C * LD;
    uint16_t* Ph = V + C * LD;
    uint16_t* Pl = Ph + C * LDP;
    float* bs = reinterpret_cast<float*>(SUMMARY ? V + C * LD : Pl + C * LDP);  // beta[64], then b_C
    float* wo = bs + C + 4;                                                      // e^{b_C - beta}[64]
    uint16_t* stage = Q;
    uint16_t* V2 = reinterpret_cast<uint16_t*>(smem + walk_lds(SUMMARY));  // VSPLIT only
    static_assert(!VSPLIT || SUMMARY, "two value planes: summary pass only");

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), n = lane & 31, half = lane >> 5;
    const SeqWalk walk = seq_walk(d, seq);
    const int nsq = (walk.n + a.m - 1) / a.m;  // segments of this sequence
    const int kbeg = seg * a.m, kend = min(walk.n, kbeg + a.m), cnt = kend - kbeg;
    const bool empty_seq = walk.n == 0 && seg == 0;  // packed input: the state passes through
    if (SUMMARY) {
        // only segments whose end state another segment starts from
        if (cnt <= 0 || (REV ? seg < a.skip : seg >= nsq - 1)) return;
    } else if (cnt <= 0 && !empty_seq) {
        return;
    }
    const bool last = empty_seq || (REV ? seg == 0 : seg == nsq - 1);  // this walk ends the sequence

    f32x16 S[4];
    _Pragma("unroll") for (int ib = 0; ib < 4; ++ib) S[ib] = f32x16{0};
    if (!SUMMARY) {
        if (a.nseg > 1) walk_state_load(S, a.bound + (size_t(seq) * a.nseg + seg) * D * D, false, wave, n, half);
        else if (a.edge_in) walk_state_load(S, a.edge_in + edge_off(d, seq), false, wave, n, half, D * d.vm);
    }

    TileRegs rq, rk, rv, rv2;
    float gval = 0.f, gtot = 0.f;
    // The summary pass visits the chunks of its segment in the order opposite to the walk (a sum: each
    // chunk's weights carry the decay of the chunks that follow it in walk order), so that the walker,
    // which runs next, starts with the rows read last.
    auto chunk_of = [&](int kk) { return (REV != SUMMARY) ? kend - 1 - kk : kbeg + kk; };
    auto gload = [&](int kk) {
        const ChunkPos p = walk_pos(d, walk, chunk_of(min(kk, cnt - 1)));
        if (DEC) {
            const int row = min(lane, p.L - 1), tok = REV ? p.L - 1 - row : row;
            gval = a.g[d.kind == 1 ? size_t(walk.bh % d.H) : p.tok0 + size_t(tok) * p.ts];
        }
        if (!SUMMARY) walk_gload<REV, kThreads>(rq, a.xq, p.tok0, p.ts, p.L, tid);
        walk_gload<REV, kThreads>(rk, a.xk, p.tok0, p.ts, p.L, tid);
        walk_gload<REV, kThreads>(rv, a.xv, p.vtok0, p.vts, p.L, tid);
        if (VSPLIT) walk_gload<REV, kThreads>(rv2, a.xv_lo, p.vtok0, p.vts, p.L, tid);
    };
    if (cnt > 0) gload(0);

    for (int kk = 0; kk < cnt; ++kk) {
        const ChunkPos cp = walk_pos(d, walk, chunk_of(kk));
        const int L = cp.L;
        // ---- registers of this chunk -> LDS; decay tables; loads of the next chunk
        if (!SUMMARY) walk_commit<kThreads>(Q, rq, L, tid);
        walk_commit<kThreads>(K, rk, L, tid);
        walk_commit<kThreads>(V, rv, L, tid);
        if (VSPLIT) walk_commit<kThreads>(V2, rv2, L, tid);
        if (DEC && wave == 0) gtot += walk_decay_tables<REV>(gval, L, SUMMARY ? gtot : 0.f, bs, wo, lane);
        gload(kk + 1);
        __syncthreads();  // (A) tiles and decay tables of this chunk are in LDS
        const float bC = DEC ? bs[C] : 0.f;

        if (!SUMMARY) {
            f32x16 O[2];
            walk_inter<DEC>(O, S, Q, bs, n, half);
            walk_scores<DEC>(K, Q, Ph, Pl, bs, wave, n, half);
            __syncthreads();  // (C) scores are in LDS; nobody reads Q any more
            _Pragma("unroll") for (int jb = 0; jb < 2; ++jb) {
                walk_intra(O[jb], jb, V, Ph, Pl, wave, lane, n, half);
                store_packed(stage, LD, 32 * jb + n, 32 * wave, half, pack_block(O[jb]));
            }
        }
        if (VSPLIT) walk_update_vsplit<DEC, !SUMMARY>(S, K, V, V2, wo, bC, wave, lane, half);
        else walk_update<DEC, !SUMMARY>(S, K, V, wo, bC, wave, lane, half);
        __syncthreads();  // (D) the output stage is complete and every read of this chunk's tiles is done
        // every thread reads back exactly the stage pieces that its own next walk_commit overwrites: no barrier
        if (!SUMMARY) walk_store<REV>(a.out, stage, cp.vtok0, cp.vts, L, tid);
    }

    // ---- the state this walk ends with
    if (SUMMARY) {
        walk_state_store(S, a.bound + (size_t(seq) * a.nseg + (REV ? seg - 1 : seg + 1)) * D * D, false, wave, n, half);
        if (tid == 0) a.gseg[size_t(seq) * a.nseg + seg] = gtot;
        return;
    }
    if (last && a.edge_out) walk_state_store(S, a.edge_out + edge_off(d, seq), false, wave, n, half, D * d.vm);
}

// forward walker, or the summary pass of either direction (grid: segments x sequences)
template <bool REV, bool DEC, bool SUMMARY, bool VSPLIT = false>
__global__ __launch_bounds__(kThreads, 2) void mk_walk(Dims d, WalkArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    walk_body<REV, DEC, SUMMARY, VSPLIT>(d, a, blockIdx.y, blockIdx.x, smem);
}

// ---------------------------------------------------------------------------------------------
// Gradient walker: dq, dk, dv and the decay gradient of a segment of chunks in one pass, forward in
// time, with the state S (as S^T: rows v, columns i) in accumulators and the state gradients dS read
// from memory, one per chunk (written by the reverse scan, fragment-major bf16).  Per chunk, with
// S = state at the chunk start, dS = gradient of the state at the chunk end, D_jr = e^{b_j-b_r} (r <= j):
//   G = (dO V^T) * D ,  As = (Q K^T) * D
//   dq^T[i][j] = e^{b_j}     sum_v S[i][v]  d_o_j[v] + sum_r K^T[i][r] G[j][r]
//   dk^T[i][r] = e^{b_C-b_r} sum_v dS[i][v] v_r[v]   + sum_j Q^T[i][j] G[j][r]
//   dv^T[v][r] = e^{b_C-b_r} sum_i dS^T[v][i] k_r[i] + sum_j dO^T[v][j] As[j][r]
//   S   <- e^{b_C} S + sum_r e^{b_C-b_r} k_r^T v_r
//   dg_t = sum_{u>=t} (q_u.dq_u - k_u.dk_u) + <S, dS>      (S after the update: the state at the chunk end)
// S enters its product as bf16 head + remainder taken from the fp32 accumulators, so the q.dq term of the decay
// gradient sees no state rounding.  G and As are each computed once per workgroup, one wave per 32 x 32 block, and
// parked as head + remainder in areas of their own; the dS rows, which arrive as the A operands of the dk inter part,
// also go to LDS for the contractions over i.  One workgroup per compute unit, four barriers per chunk.
// LDS: Q | K | V | dO (64 x LD; at the end the stages of dq, dk, dv) | G head | G remainder | As head |
//      As remainder (64 x LDP each) | dS rows (128 x LD) | bs | wo | red (4 x 2 x 64) | zred
constexpr int kWalkGradLds = (4 * C * LD + 4 * C * LDP + D * LD) * 2 + (2 * C + 8) * 4 + 4 * 64 * 2 * 4 + 64;

struct GradArgs {
    const uint16_t *q, *k, *v, *d_o;
    const float* g;
    const uint16_t* dstates;  // [BH*N] fragment-major bf16: slot c = gradient of the state at the end of chunk c
    uint16_t *dq, *dk, *dv;
    float* dg_tok;            // per-token scalar kind: d_log_decay itself; per-head kind: [BH*N] per-chunk sums
    const float* edge_in;     // M_0 [i][v] per sequence or NULL
    const float* bound;       // entry states of the segments ([i][v]) when nseg > 1
    int m, nseg;
    const uint16_t* v_lo;     // VSPLIT: remainder plane of the values (same layout as v)
    // VSPLIT: dU (head, remainder; [BH*T][128] in the library's own order) and the product dW = -dU S^T of every chunk with
    // the state it starts from (head, remainder, same order)
    const uint16_t *du_h, *du_l;
    uint16_t *dw_h, *dw_l;
    // the entry states may be kept at a finer grain than this walk's segments: bound holds bound_n slots per sequence,
    // one per m / bound_per chunks, and segment s enters with slot s * bound_per (0: same grain, nseg slots)
    int bound_per, bound_n;
    // d_v = 256 (two passes, one per 128-wide value slice; dq and dk sum over them): the first pass leaves its dq and dk as
    // bf16 head + remainder in these four planes ([BH*T][128], library order: dq head, dq remainder, dk head, dk remainder),
    // the second adds them to its own before the one rounding
    uint16_t* part[4];
};
// VSPLIT (the delta-rule backward, whose values are the pseudo-values U = head + remainder): the values enter
// every product with both planes; the value gradient is not formed (it is the caller's dU once more) and its
// output receives the remainder of the key gradient instead (dk = head, dv = remainder).  The area of the dS rows
// holds the two planes of dU instead, and the walker also leaves dW = -dU S^T (the gradient of the delta rule's
// What), staged through the d_o tile and the second value tile.
__host__ __device__ constexpr int walk_grad_lds(bool vsplit) { return kWalkGradLds + (vsplit ? C * LD * 2 : 0); }

// inter product of the state with rows kept in two planes (head Qh, remainder Ql), the state blocks converted once:
// O^T[i][t] = sum_v S[i][v] (Qh + Ql)[t][v], remainder x remainder left out
__device__ __forceinline__ void walk_inter_split(f32x16 (&O)[2], const f32x16 (&S)[4], const uint16_t* Qh, const uint16_t* Ql, int n,
                                                 int half) {
    O[0] = f32x16{0};
    O[1] = f32x16{0};
    _Pragma("unroll") for (int ib = 0; ib < 4; ++ib)
        _Pragma("unroll") for (int p = 0; p < 2; ++p) {
            u32x4 hi, lo;
            _Pragma("unroll") for (int e = 0; e < 4; ++e) {
                const float x0 = S[ib][8 * p + 2 * e], x1 = S[ib][8 * p + 2 * e + 1];
                hi[e] = pack2(x0, x1);
                lo[e] = pack2(x0 - bf16_lo(hi[e]), x1 - bf16_hi(hi[e]));
            }
            const bf16x8 sh = __builtin_bit_cast(bf16x8, hi), sl = __builtin_bit_cast(bf16x8, lo);
            const bf16x8 qh0 = frag_perm(Qh, LD, n, 32 * ib + 16 * p, half), qh1 = frag_perm(Qh, LD, 32 + n, 32 * ib + 16 * p, half);
            const bf16x8 ql0 = frag_perm(Ql, LD, n, 32 * ib + 16 * p, half), ql1 = frag_perm(Ql, LD, 32 + n, 32 * ib + 16 * p, half);
            O[0] = mfma(sh, qh0, O[0]);
            O[1] = mfma(sh, qh1, O[1]);
            O[0] = mfma(sl, qh0, O[0]);
            O[1] = mfma(sl, qh1, O[1]);
            O[0] = mfma(sh, ql0, O[0]);
            O[1] = mfma(sh, ql1, O[1]);
        }
}

// Gradient walker kernel: eight waves, two per SIMD.  The work of a chunk is split by function, not by data, so that
// neither group needs the other's registers:
//   waves 0..3 (wave w: key features i in [32w, 32w+32)) carry the state; they form dq (inter part from the state, intra
//              part from G), <S, dS>, with VSPLIT dW, and move the state on;
//   waves 4..7 (wave w: the same i slice for dk, value features v in [32w, 32w+32) for dv) hold the dS rows of the chunk;
//              they compute the score blocks (G, As), dk and dv.
// Each group runs a loop of its own with the same four barriers per chunk, so a SIMD always has one wave of either
// kind to issue from: the matrix, vector and LDS work of the two overlap instead of queueing behind one wave's waits.
// Plain case: all 512 threads share the tile traffic (global -> registers -> LDS, stage -> global), and the carrier
// waves read dS for <S, dS> at the (i, v) of their state registers from the LDS rows.
// VSPLIT: the carrier waves' registers are full (state, dq, dW), so the other group moves most of the tiles; the carrier
// waves form <S, dS> (dS by loads of their own from the fragment-major array, which the other group has just pulled
// into L2: the LDS area of the dS rows holds dU) and dW before barrier (2), and dq and the state update after it, so
// that the accumulators of dW and dq never coexist.
constexpr int kGrad8Threads = 512;

// WIDE: 0 the only pass; 1 the first of two value-slice passes (dq, dk to the partial planes); 2 the second
template <bool DEC, bool WANT_DG, bool VSPLIT = false, int WIDE = 0>
__global__ __launch_bounds__(kGrad8Threads, 1) void mk_walk_grad(Dims d, GradArgs a) {
    static_assert(!(VSPLIT && WIDE), "the two-plane case has 128 value columns");
    extern __shared__ __align__(16) unsigned char smem[];
    uint16_t* Q = reinterpret_cast<uint16_t*>(smem);
    uint16_t* K = Q + C * LD;
    uint16_t* V = K + C * LD;
    uint16_t* dO = V + C * LD;
    uint16_t* Gh = dO + C * LD;
    uint16_t* Gl = Gh + C * LDP;
    uint16_t* Ah = Gl + C * LDP;
    uint16_t* Al = Ah + C * LDP;
    uint16_t* dSt = Al + C * LDP;    // [i][v] rows of dS, all 128
    float* bs = reinterpret_cast<float*>(dSt + D * LD);
    float* wo = bs + C + 4;
    float* red = wo + C + 4;         // [i slice][2][64]: q.dq, k.dk partial sums over the slice
    float* zred = red + 4 * 2 * 64;  // [i slice]: partial <S, dS>
    uint16_t* V2 = reinterpret_cast<uint16_t*>(smem + kWalkGradLds);  // VSPLIT only
    uint16_t* dUh = dSt;             // VSPLIT: 64 x LD each, over the dS rows
    uint16_t* dUl = dSt + C * LD;
    uint16_t* Wl = Ah;               // VSPLIT (no As): stage of the remainder plane of dW, 64 x LD
    uint16_t* Lq = Gh;               // WIDE == 1: stages of the remainder planes of dq and dk (G and As are spent after (3))
    uint16_t* Lk = Ah;
    static_assert(2 * C * LDP >= C * LD, "a 64 x LD stage fits the area of G");
    static_assert(2 * C * LDP >= C * LD, "the dW stage fits the area of As");
    constexpr int NT = VSPLIT ? 256 : kGrad8Threads;  // threads that share the tile traffic

    const int seq = blockIdx.y, seg = blockIdx.x;
    // the wave index as a scalar: the branch between the two groups is then a scalar branch (each group's barriers are
    // executed by its own waves only, whatever the compiler makes of the vector condition), and 32 * wave offsets are scalars
    const int tid = threadIdx.x, wave8 = __builtin_amdgcn_readfirstlane(tid >> 6), wave = wave8 & 3;
    int lane = tid & 63, n = lane & 31, half = lane >> 5;
    int tt = VSPLIT ? tid & 255 : tid;  // index among the threads that move tiles
    const bool carrier = wave8 < 4;     // waves 0..3
    // VSPLIT: every LDS access pattern keeps a lane-dependent base address per 64 KiB window of the 159 KiB
    // in use, and with the state, two sets of accumulators and the tiles in flight there is no room to keep a hundred of
    // them alive across the loop.  Hiding the lane id from the optimiser at the phase boundaries makes it recompute the
    // addresses of a phase inside the phase (a few vector instructions each) instead of spilling them.
    auto fresh = [&]() {
        if (VSPLIT) {
            asm volatile("" : "+v"(lane));
            n = lane & 31;
            half = lane >> 5;
            tt = 64 * wave + lane;
        }
    };
    const SeqWalk walk = seq_walk(d, seq);
    const int kbeg = seg * a.m, kend = min(walk.n, kbeg + a.m), cnt = kend - kbeg;
    if (cnt <= 0) return;

    // VSPLIT: the carrier group moves the head plane of dU in, and d_o when it has no decay tables to keep (measured:
    // with them it is the slower group already); the other group moves the other tiles in and all but the head of dW out
    constexpr bool kCarrierMovesDo = !DEC;
    TileRegs tq, tk, tv, to, tv2, tdh, tdl;
    auto gload_tiles = [&](const ChunkPos& p, bool first_group) {
        if (!VSPLIT || !first_group) {
            walk_gload<false, NT>(tq, a.q, p.tok0, p.ts, p.L, tt);
            walk_gload<false, NT>(tk, a.k, p.tok0, p.ts, p.L, tt);
            walk_gload<false, NT>(tv, a.v, p.vtok0, p.vts, p.L, tt);
        }
        if (!VSPLIT || first_group == kCarrierMovesDo) walk_gload<false, NT>(to, a.d_o, p.vtok0, p.vts, p.L, tt);
        if (VSPLIT && first_group) walk_gload<false, NT>(tdh, a.du_h, p.wtok0, 1, p.L, tt);
        if (VSPLIT && !first_group) {
            walk_gload<false, NT>(tv2, a.v_lo, p.vtok0, p.vts, p.L, tt);
            walk_gload<false, NT>(tdl, a.du_l, p.wtok0, 1, p.L, tt);
        }
    };
    auto commit_tiles = [&](int L, bool first_group) {
        if (!VSPLIT || !first_group) {
            walk_commit<NT>(Q, tq, L, tt);
            walk_commit<NT>(K, tk, L, tt);
            walk_commit<NT>(V, tv, L, tt);
        }
        if (!VSPLIT || first_group == kCarrierMovesDo) walk_commit<NT>(dO, to, L, tt);
        if (VSPLIT && first_group) walk_commit<NT>(dUh, tdh, L, tt);
        if (VSPLIT && !first_group) {
            walk_commit<NT>(V2, tv2, L, tt);
            walk_commit<NT>(dUl, tdl, L, tt);
        }
    };
    auto store_tiles = [&](const ChunkPos& cp, bool first_group) {
        // Every thread reads back exactly the stage pieces that its own next commit overwrites: no barrier between this and
        // the next chunk's commit.  (VSPLIT: the head of dW is staged over the plane of dU that the carrier group commits,
        // so that group stores it; the stage of the remainder is next written after barrier (1).)
        if (!VSPLIT || !first_group) {
            if (WIDE == 1) {  // head and remainder of this pass's dq and dk, for the second pass
                walk_store<false, NT>(a.part[0], Q, cp.wtok0, 1, cp.L, tt);
                walk_store<false, NT>(a.part[1], Lq, cp.wtok0, 1, cp.L, tt);
                walk_store<false, NT>(a.part[2], K, cp.wtok0, 1, cp.L, tt);
                walk_store<false, NT>(a.part[3], Lk, cp.wtok0, 1, cp.L, tt);
            } else {
                walk_store<false, NT>(a.dq, Q, cp.tok0, cp.ts, cp.L, tt);
                walk_store<false, NT>(a.dk, K, cp.tok0, cp.ts, cp.L, tt);
            }
            walk_store<false, NT>(a.dv, V, cp.vtok0, cp.vts, cp.L, tt);
        }
        if (VSPLIT && first_group) walk_store<false, NT>(a.dw_h, dUh, cp.wtok0, 1, cp.L, tt);
        if (VSPLIT && !first_group) walk_store<false, NT>(a.dw_l, Wl, cp.wtok0, 1, cp.L, tt);
    };
    // WIDE == 2: the first pass's share of a gradient block (lane = token 32 nb + n, registers = this wave's 32 features)
    struct Part { u32x2 h[4], l[4]; };
    auto part_load = [&](Part& pt, const uint16_t* ph, const uint16_t* pl, const ChunkPos& cp, int nb) {
        const size_t row = (cp.wtok0 + size_t(min(32 * nb + n, max(cp.L, 1) - 1))) * D + 32 * wave + 4 * half;
        _Pragma("unroll") for (int g = 0; g < 4; ++g) {
            pt.h[g] = *reinterpret_cast<const u32x2*>(ph + row + 8 * g);
            pt.l[g] = *reinterpret_cast<const u32x2*>(pl + row + 8 * g);
        }
    };
    auto part_add = [](f32x16& x, const Part& pt) {
        _Pragma("unroll") for (int g = 0; g < 4; ++g) {
            x[4 * g + 0] += bf16_lo(pt.h[g].x) + bf16_lo(pt.l[g].x);
            x[4 * g + 1] += bf16_hi(pt.h[g].x) + bf16_hi(pt.l[g].x);
            x[4 * g + 2] += bf16_lo(pt.h[g].y) + bf16_lo(pt.l[g].y);
            x[4 * g + 3] += bf16_hi(pt.h[g].y) + bf16_hi(pt.l[g].y);
        }
    };
    // head of a block; the block keeps its remainder
    auto split_block = [](f32x16& x) {
        const PackedBlock h = pack_block(x);
        _Pragma("unroll") for (int g = 0; g < 4; ++g) {
            x[4 * g + 0] -= bf16_lo(h.v[g].x);
            x[4 * g + 1] -= bf16_hi(h.v[g].x);
            x[4 * g + 2] -= bf16_lo(h.v[g].y);
            x[4 * g + 3] -= bf16_hi(h.v[g].y);
        }
        return h;
    };

    if (carrier) {
        // S block vb of this wave: S[vb][4g+j] = M[i = 32 wave + n][v = 32 vb + 8g + 4 half + j]
        f32x16 S[4];
        _Pragma("unroll") for (int vb = 0; vb < 4; ++vb) S[vb] = f32x16{0};
        {
            if (a.nseg > 1)
                walk_state_load(S, a.bound + (size_t(seq) * (a.bound_per ? a.bound_n : a.nseg) + seg * (a.bound_per ? a.bound_per : 1)) * D * D,
                                true, wave, n, half);
            else if (a.edge_in) walk_state_load(S, a.edge_in + edge_off(d, seq), true, wave, n, half, D * d.vm);
        }
        float gval = 0.f;
        auto gload = [&](int kk) {
            const ChunkPos p = walk_pos(d, walk, kbeg + min(kk, cnt - 1));
            if (DEC) gval = a.g[d.kind == 1 ? size_t(walk.bh % d.H) : p.tok0 + size_t(min(lane, p.L - 1)) * p.ts];
            gload_tiles(p, true);
        };
        // dq^T[i][j] += sum_{r<=j} K^T[i][r] G[j][r] (keys r >= 32 never reach queries j < 32), its share of the decay gradient
        auto dq_intra = [&](f32x16 (&aq)[2], PackedBlock (&resq)[2], PackedBlock (&resql)[2], const ChunkPos& cp) {
            Part pt[2];
            if (WIDE == 2) {
                part_load(pt[0], a.part[0], a.part[1], cp, 0);
                part_load(pt[1], a.part[0], a.part[1], cp, 1);
            }
            _Pragma("unroll") for (int nb = 0; nb < 2; ++nb) {
                const int tok = 32 * nb + n;
                _Pragma("unroll") for (int ks = 0; ks < 2 * (nb + 1); ++ks) {
                    const bf16x8 kt = frag_tr(K, LD, 16 * ks, 32 * wave, lane);
                    aq[nb] = mfma(kt, frag(Gh, LDP, tok, 16 * ks + 8 * half), aq[nb]);
                    aq[nb] = mfma(kt, frag(Gl, LDP, tok, 16 * ks + 8 * half), aq[nb]);
                }
                if (WANT_DG) {
                    float pq = row_dot(Q, tok, wave, half, aq[nb]);
                    pq += __shfl_xor(pq, 32, 64);
                    if (half == 0) red[(wave * 2 + 0) * 64 + tok] = pq;
                }
                if (WIDE == 2) part_add(aq[nb], pt[nb]);  // after the decay gradient took this pass's own share
                if (WIDE == 1) {
                    resq[nb] = split_block(aq[nb]);
                    resql[nb] = pack_block(aq[nb]);
                } else {
                    resq[nb] = pack_block(aq[nb]);
                }
            }
        };
        // <S, dS> with the state at the END of the chunk, over this wave's rows i: together with the running sums of
        // q.dq - k.dk this is the whole decay gradient (<e^{b_C} S + S_chunk, dS> = e^{b_C} <S, dS> + sum_r k_r.dk_r^{inter}).
        // dS at the (i, v) of the state registers: from the LDS rows, or (VSPLIT) from the registers dsz
        auto state_dot = [&](const u32x2 (&dsz)[16]) {
            float z = 0.f;
            _Pragma("unroll") for (int vb = 0; vb < 4; ++vb)
                _Pragma("unroll") for (int g = 0; g < 4; ++g) {
                    const u32x2 x = VSPLIT ? dsz[4 * vb + g]
                                           : *reinterpret_cast<const u32x2*>(dSt + (32 * wave + n) * LD + 32 * vb + 8 * g + 4 * half);
                    z += S[vb][4 * g] * bf16_lo(x.x) + S[vb][4 * g + 1] * bf16_hi(x.x) + S[vb][4 * g + 2] * bf16_lo(x.y) +
                         S[vb][4 * g + 3] * bf16_hi(x.y);
                }
            for (int off = 32; off > 0; off >>= 1) z += __shfl_xor(z, off, 64);
            if (lane == 0) zred[wave] = z;
        };
        gload(0);
        for (int kk = 0; kk < cnt; ++kk) {
            const ChunkPos cp = walk_pos(d, walk, kbeg + kk);
            const int L = cp.L;
            fresh();
            commit_tiles(L, true);
            if (DEC && wave8 == 0) walk_decay_tables<false>(gval, L, 0.f, bs, wo, lane);
            __syncthreads();  // (1) tiles, dS rows and decay tables of this chunk are in LDS
            fresh();
            const float bC = DEC ? bs[C] : 0.f;
            f32x16 aq[2];
            PackedBlock resw[2], resq[2], resql[2];
            if (VSPLIT) {
                // dW^T[i][t] = -sum_v S[i][v] dU[t][v]; the remainder plane is staged at once (nobody else uses its area)
                f32x16 dw[2];
                walk_inter_split(dw, S, dUh, dUl, n, half);
                _Pragma("unroll") for (int nb = 0; nb < 2; ++nb) {
                    _Pragma("unroll") for (int x = 0; x < 16; ++x) dw[nb][x] = -dw[nb][x];
                    resw[nb] = split_block(dw[nb]);
                    store_packed(Wl, LD, 32 * nb + n, 32 * wave, half, pack_block(dw[nb]));
                }
            } else {
                walk_inter<DEC>(aq, S, dO, bs, n, half);
            }
            u32x2 dsz[16];  // VSPLIT: dS at the (i, v) of the state registers, four consecutive v per load
            if (!VSPLIT) {
                // the state moves on to the end of the chunk (roles: key = v, value = k)
                walk_update<DEC, true>(S, V, K, wo, bC, wave, lane, half);
                if (WANT_DG) state_dot(dsz);
                if (kk + 1 < cnt) gload(kk + 1);
            }
            __syncthreads();  // (2) G and As are in LDS
            fresh();
            if (VSPLIT) {
                // the planes of dU are dead: the head of dW is staged over the first
                _Pragma("unroll") for (int nb = 0; nb < 2; ++nb) store_packed(dUh, LD, 32 * nb + n, 32 * wave, half, resw[nb]);
                walk_inter<DEC>(aq, S, dO, bs, n, half);
                dq_intra(aq, resq, resql, cp);
                fresh();
                if (WANT_DG) {
                    const uint16_t* dS = a.dstates + cp.slot * D * D;
                    _Pragma("unroll") for (int vb = 0; vb < 4; ++vb)
                        _Pragma("unroll") for (int g = 0; g < 4; ++g)
                            dsz[4 * vb + g] = *reinterpret_cast<const u32x2*>(dS + state_frag_off(wave, 2 * vb + (g >> 1), 32 * (g & 1) + n) + 4 * half);
                }
                walk_update<DEC, true, true>(S, V, K, wo, bC, wave, lane, half, V2);
                if (WANT_DG) state_dot(dsz);
                if (kk + 1 < cnt) gload(kk + 1);
            } else {
                dq_intra(aq, resq, resql, cp);
            }
            __syncthreads();  // (3) every wave is done with the tiles
            fresh();
            _Pragma("unroll") for (int nb = 0; nb < 2; ++nb) {
                store_packed(Q, LD, 32 * nb + n, 32 * wave, half, resq[nb]);
                if (WIDE == 1) store_packed(Lq, LD, 32 * nb + n, 32 * wave, half, resql[nb]);
            }
            __syncthreads();  // (4)
            fresh();
            store_tiles(cp, true);
            if (WANT_DG && wave8 == 0) {
                // fixed-order sums over the four feature slices, then the reverse in-chunk running sum
                float w = 0.f;
                const float z = (zred[0] + zred[1]) + (zred[2] + zred[3]);
                _Pragma("unroll") for (int wv = 0; wv < 4; ++wv) w += red[(wv * 2 + 0) * 64 + tid] - red[(wv * 2 + 1) * 64 + tid];
                float sfx = w;  // suffix sum of w over tokens >= tid
                for (int off = 1; off < 64; off <<= 1) {
                    const float y = __shfl_down(sfx, off, 64);
                    if (tid + off < 64) sfx += y;
                }
                float dgv = tid < L ? sfx + z : 0.f;
                constexpr bool add = WIDE == 2;  // the decay gradient sums over the value slices too
                if (d.kind == 1) {
                    // one decay per head: only the sum over tokens is wanted; this chunk's share, in a fixed order
                    for (int off = 32; off > 0; off >>= 1) dgv += __shfl_xor(dgv, off, 64);
                    if (tid == 0) a.dg_tok[cp.slot] = add ? a.dg_tok[cp.slot] + dgv : dgv;
                } else if (tid < L) {
                    float* pg = a.dg_tok + cp.tok0 + size_t(tid) * cp.ts;
                    *pg = add ? *pg + dgv : dgv;
                }
            }
        }
    } else {
        bf16x8 dsfrag[8];
        auto gload = [&](int kk) {
            const ChunkPos p = walk_pos(d, walk, kbeg + min(kk, cnt - 1));
            gload_tiles(p, false);
            // rows i in [32w, 32w+32) of dS: A operands [m = i][k = v]
            const uint16_t* dS = a.dstates + p.slot * D * D;
            _Pragma("unroll") for (int ks = 0; ks < 8; ++ks)
                dsfrag[ks] = __builtin_nontemporal_load(reinterpret_cast<const bf16x8*>(dS + state_frag_off(wave, ks, lane)));
        };
        // one 32 x 32 score block (0: (0,0), 1: (1,0), 2: (1,1)), mask and decay on its accumulators, as head + remainder
        auto score = [&](bool isG, int bi) {
            const int pjb = bi ? 1 : 0, prb = bi == 2 ? 1 : 0;
            // D[m = r][n = j] = v_r . d_o_j  or  k_r . q_j
            f32x16 P = isG ? score_block2(V, 32 * prb, dO, 32 * pjb, n, half) : score_block2(K, 32 * prb, Q, 32 * pjb, n, half);
            if (VSPLIT && isG) P = score_block2(V2, 32 * prb, dO, 32 * pjb, n, half, P);
            walk_mask<DEC>(P, 32 * prb, 32 * pjb + n, bs, half);
            store_block_t_split(isG ? Gh : Ah, isG ? Gl : Al, LDP, 32 * pjb + n, 32 * prb, half, P);
        };
        gload(0);
        for (int kk = 0; kk < cnt; ++kk) {
            const ChunkPos cp = walk_pos(d, walk, kbeg + kk);
            const int L = cp.L;
            fresh();
            commit_tiles(L, false);
            if (!VSPLIT) {
                // the dS rows of this wave, for the contractions over i (dv, <S, dS>)
                _Pragma("unroll") for (int ks = 0; ks < 8; ++ks)
                    *reinterpret_cast<bf16x8*>(dSt + (32 * wave + n) * LD + 16 * ks + 8 * half) = dsfrag[ks];
            }
            __syncthreads();  // (1)
            fresh();
            // G = (dO V^T) * D first (the other group waits for it at (2)), then As = (Q K^T) * D, which only dv needs
            if (VSPLIT) {
                if (wave < 3) score(true, wave);
            } else {
                if (wave < 3) score(true, wave);
                else score(false, 0);
                if (wave < 2) score(false, wave + 1);
            }
            // inter parts: dk^T[i][r] from the dS rows in registers, dv^T[v][r] from the transposed read of the LDS rows
            f32x16 ak[2] = {{0}, {0}}, av[2] = {{0}, {0}};
            _Pragma("unroll") for (int nb = 0; nb < 2; ++nb) {
                const int tok = 32 * nb + n;
                _Pragma("unroll") for (int ks = 0; ks < 8; ++ks) ak[nb] = mfma(dsfrag[ks], frag(V, LD, tok, 16 * ks + 8 * half), ak[nb]);
                if (VSPLIT) {
                    _Pragma("unroll") for (int ks = 0; ks < 8; ++ks) ak[nb] = mfma(dsfrag[ks], frag(V2, LD, tok, 16 * ks + 8 * half), ak[nb]);
                }
                if (DEC) {
                    const float wk = wo[tok];
                    _Pragma("unroll") for (int x = 0; x < 16; ++x) ak[nb][x] *= wk;
                }
            }
            if (kk + 1 < cnt) gload(kk + 1);  // the dS registers are free
            if (!VSPLIT) {
                _Pragma("unroll") for (int ks = 0; ks < 8; ++ks) {
                    const bf16x8 dst = frag_tr(dSt, LD, 16 * ks, 32 * wave, lane);  // dS^T[v][i], i = 16 ks + ..
                    _Pragma("unroll") for (int nb = 0; nb < 2; ++nb)
                        av[nb] = mfma(dst, frag(K, LD, 32 * nb + n, 16 * ks + 8 * half), av[nb]);
                }
                if (DEC) {
                    _Pragma("unroll") for (int nb = 0; nb < 2; ++nb) {
                        const float wk = wo[32 * nb + n];
                        _Pragma("unroll") for (int x = 0; x < 16; ++x) av[nb][x] *= wk;
                    }
                }
            }
            __syncthreads();  // (2) G and As are in LDS
            fresh();
            PackedBlock resk[2], resv[2], reskl[2];
            Part pt[2];
            if (WIDE == 2) {
                part_load(pt[0], a.part[2], a.part[3], cp, 0);
                part_load(pt[1], a.part[2], a.part[3], cp, 1);
            }
            _Pragma("unroll") for (int nb = 0; nb < 2; ++nb) {
                const int tok = 32 * nb + n;
                // dk^T[i][r] += sum_{j>=r} Q^T[i][j] G[j][r]: queries j < 32 never see keys r >= 32
                _Pragma("unroll") for (int ks = 2 * nb; ks < 4; ++ks) {
                    const bf16x8 qt = frag_tr(Q, LD, 16 * ks, 32 * wave, lane);
                    ak[nb] = mfma(qt, frag_tr(Gh, LDP, 16 * ks, 32 * nb, lane), ak[nb]);  // B[k = j][n = r] = G[j][r]
                    ak[nb] = mfma(qt, frag_tr(Gl, LDP, 16 * ks, 32 * nb, lane), ak[nb]);
                }
                if (WANT_DG) {
                    float pk = row_dot(K, tok, wave, half, ak[nb]);
                    pk += __shfl_xor(pk, 32, 64);
                    if (half == 0) red[(wave * 2 + 1) * 64 + tok] = pk;
                }
                if (VSPLIT) {  // the key gradient leaves as head + remainder (the caller adds to it before rounding)
                    resk[nb] = split_block(ak[nb]);
                    resv[nb] = pack_block(ak[nb]);
                } else {
                    if (WIDE == 2) part_add(ak[nb], pt[nb]);
                    if (WIDE == 1) {
                        resk[nb] = split_block(ak[nb]);
                        reskl[nb] = pack_block(ak[nb]);
                    } else {
                        resk[nb] = pack_block(ak[nb]);
                    }
                    // dv^T[v][r] += sum_{j>=r} dO^T[v][j] As[j][r]
                    _Pragma("unroll") for (int ks = 2 * nb; ks < 4; ++ks) {
                        const bf16x8 dot = frag_tr(dO, LD, 16 * ks, 32 * wave, lane);
                        av[nb] = mfma(dot, frag_tr(Ah, LDP, 16 * ks, 32 * nb, lane), av[nb]);  // B[k = j][n = r] = As[j][r]
                        av[nb] = mfma(dot, frag_tr(Al, LDP, 16 * ks, 32 * nb, lane), av[nb]);
                    }
                    resv[nb] = pack_block(av[nb]);
                }
            }
            __syncthreads();  // (3)
            fresh();
            _Pragma("unroll") for (int nb = 0; nb < 2; ++nb) {
                store_packed(K, LD, 32 * nb + n, 32 * wave, half, resk[nb]);
                store_packed(V, LD, 32 * nb + n, 32 * wave, half, resv[nb]);
                if (WIDE == 1) store_packed(Lk, LD, 32 * nb + n, 32 * wave, half, reskl[nb]);
            }
            __syncthreads();  // (4)
            fresh();
            store_tiles(cp, false);
        }
    }
}

// Entry state of every segment from the segments' own contributions (left by the summary pass in the
// slot of the segment that follows in walk order) and total log-decays: E' = e^{G} E + U, in walk order.
// grid: (128 * 128 / 256, seqs)
template <bool REV>
__global__ __launch_bounds__(kThreads) void mk_bound_scan(Dims d, const float* __restrict__ edge_in, float* __restrict__ bound,
                                                          const float* __restrict__ gseg, int m, int nseg, int skip) {
    const int seq = blockIdx.y, e = blockIdx.x * kThreads + threadIdx.x;
    const SeqWalk walk = seq_walk(d, seq);
    const int nsq = max(1, (walk.n + m - 1) / m);
    float* b = bound + size_t(seq) * nseg * D * D + e;
    const float* gs = gseg + size_t(seq) * nseg;
    float E = edge_in ? edge_in[edge_off(d, seq) + size_t(e / D) * D * d.vm + e % D] : 0.f;
    // The contributions are read eight segments at a time before any of them is replaced: the reads of a batch do not
    // depend on each other, only the recurrence does (read - update - write in turn pays one memory latency per segment).
    constexpr int G = 8;
    if (!REV) {
        b[0] = E;
        for (int s0 = 0; s0 + 1 < nsq; s0 += G) {
            float u[G], w[G];
            _Pragma("unroll") for (int i = 0; i < G; ++i) {
                const int s = min(s0 + i, nsq - 2);
                u[i] = b[size_t(s + 1) * D * D];
                w[i] = gs[s];
            }
            _Pragma("unroll") for (int i = 0; i < G; ++i)
                if (s0 + i + 1 < nsq) {
                    E = __expf(w[i]) * E + u[i];
                    b[size_t(s0 + i + 1) * D * D] = E;
                }
        }
    } else {
        b[size_t(nsq - 1) * D * D] = E;
        for (int s0 = nsq - 1; s0 >= skip; s0 -= G) {  // slots below skip - 1 are entered by no walk
            float u[G], w[G];
            _Pragma("unroll") for (int i = 0; i < G; ++i) {
                const int s = max(s0 - i, skip);
                u[i] = b[size_t(s - 1) * D * D];
                w[i] = gs[s];
            }
            _Pragma("unroll") for (int i = 0; i < G; ++i)
                if (s0 - i >= skip) {
                    E = __expf(w[i]) * E + u[i];
                    b[size_t(s0 - i - 1) * D * D] = E;
                }
        }
    }
}

