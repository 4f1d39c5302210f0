// Fused chunk walkers of the scalar decay kinds (none / per head / per token): bf16 operands, fp32
// accumulation, chunk = 64, d_k = d_v = 128.  Included by lsm_mfma.hip.
//
// One workgroup walks a run of consecutive chunks (a "segment") of one (b,h) recurrence with the
// 128 x 128 state in MFMA accumulators, so no per-chunk state ever goes to memory.  Per chunk it
// evaluates Algorithm 2 of the paper with the decay folded in,
//     out_t = e^{beta_t} x^q_t S + sum_{r <= t} (x^q_t . x^k_r) e^{beta_t - beta_r} x^v_r      (O_inter + O_intra)
//     S    <- e^{b_C} S + sum_r e^{b_C - beta_r} x^k_r^T x^v_r                                (chunk state, prefix)
// for three row tensors in the roles "query", "key", "value".  The same body serves all four outputs:
//     o   : forward in time,  roles (q, k, v),    S = M
//     dq  : forward in time,  roles (d_o, v, k),  S = M^T
//     dv  : backward in time, roles (k, q, d_o),  S = dM
//     dk  : backward in time, roles (v, d_o, q),  S = dM^T
// since each gradient of the recurrence is again a causal (or anti-causal) linear-attention read-out.
// Walking backward, a chunk's rows are loaded in reverse token order, and beta is the exclusive instead
// of the inclusive running sum of the log-decays in walk order; everything else is identical.
//
// Segments: with fewer recurrences than the chip has compute units a sequence is cut into segments of
// m chunks.  A first pass (SUMMARY: the state update alone, from a zero state) leaves each segment's
// own contribution and total log-decay, a small scan turns them into the state every segment starts
// from, and the walkers then run all segments in parallel.  Only those entry states (one per m chunks)
// ever reach memory.
//
// Decay gradient (DG).  With F_t = sum_{u >= t, u in chunk} q_u . dq_u,  R_t likewise with k_u . dk_u,
//     dg_t = F_t - R_t + y_{c+1} ,    y_{c+1} = <S_{c+1}, dS_{c+1}> = y_c - a_c + b_c ,
//     a_c = sum_{t in c} q_t . dq_t^{inter} ,   b_c = sum_{t in c} k_t . dk_t^{inter} ,   y_0 = <M_0, dM_0>
// (the adjoint identity dg_t = a_t <dM_t, M_{t-1}> split at the chunk boundaries).  The dq walker emits
// q_t . dq_t and a_c, the dk walker k_t . dk_t and b_c, the dv walker y_0; a small kernel combines them.
// All of them are formed from the fp32 accumulators, and the state enters its products as a bf16 head
// plus a bf16 remainder, so that the running sum over chunks does not collect the 2^-9 rounding of a
// single bf16 operand.
#pragma once

struct WalkArgs {
    const uint16_t *xq, *xk, *xv;  // rows in the query, key and value role
    const uint16_t* xx;            // DG: rows dotted with the output rows
    const float* g;                // log-decay (per kind)
    uint16_t* out;
    const float* edge_in;  // state a whole sequence starts from, [i][v] fp32 per sequence; NULL = zero
    float* edge_out;       // state it ends with; NULL = not wanted
    float* bound;          // [seqs][nseg][128 x 128] fp32, [i][v]: entry state of every segment (nseg > 1)
    float* gseg;           // [seqs][nseg]: total log-decay of each segment (SUMMARY writes)
    float* pdot;           // DG: [BH*T] x_t . out_t
    float* isum;           // DG: [BH*N] sum over the chunk of x_t . out_t^{inter}
    const float* dot_with; // if y0: [i][v] fp32 per sequence, its inner product with the final state goes to y0 (NULL: 0)
    float* y0;             // [seqs] or NULL
    int transposed;        // the walker's state [key feature][value feature] is the transpose of the [i][v] arrays
    int m, nseg;           // chunks per segment, segments per sequence (upper bound for packed input)
};

// tile rows in walk order: row r holds token r (forward) or token L-1-r (backward); rows >= L are zero
template <bool REV>
__device__ __forceinline__ void walk_gload(TileRegs& r, const uint16_t* src, size_t tok0, int ts, int L, int tid) {
    _Pragma("unroll") for (int it = 0; it < 4; ++it) {
        const int p = tid + kThreads * it, row = min(p >> 4, L - 1), cp = p & 15;
        const int tok = REV ? L - 1 - row : row;
        r.v[it] = *reinterpret_cast<const u32x4*>(src + (tok0 + size_t(tok) * ts) * D + cp * 8);
    }
}
template <bool REV>
__device__ __forceinline__ void walk_store(uint16_t* dst, const uint16_t* src, size_t tok0, int ts, int L, int tid) {
    _Pragma("unroll") for (int it = 0; it < 4; ++it) {
        const int p = tid + kThreads * it, row = p >> 4, cp = p & 15;
        if (row < L)
            __builtin_nontemporal_store(*reinterpret_cast<const u32x4*>(src + row * LD + cp * 8),
                                        reinterpret_cast<u32x4*>(dst + (tok0 + size_t(REV ? L - 1 - row : row) * ts) * D + cp * 8));
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

constexpr int kWalkTiles = 3;  // Q (later the output stage), K, V; DG adds X
__host__ __device__ constexpr int walk_lds(bool dg, bool summary) {
    return summary ? 2 * C * LD * 2 + (2 * C + 8) * 4
                   : ((dg ? 4 : 3) * C * LD + 2 * C * LDP) * 2 + (2 * C + 8) * 4 + (dg ? 4 * 2 * C * 4 : 0);
}

// REV: walk backward in time.  DEC: a decay is present.  DG: emit the dot products of the decay
// gradient (needs a.xx).  SUMMARY: the state update alone, from a zero state, result to a.bound / a.gseg.
template <bool REV, bool DEC, bool DG, bool SUMMARY>
__device__ __forceinline__ void walk_body(const Dims& d, const WalkArgs& a, int seq, int seg, unsigned char* smem) {
    // LDS: SUMMARY: K | V | bs | wo;   else: Q | K | V | (X) | P head | P remainder | bs | wo | (red)
    uint16_t* Q = reinterpret_cast<uint16_t*>(smem);
    uint16_t* K = SUMMARY ? Q : Q + C * LD;
    uint16_t* V = K + C * LD;
    uint16_t* X = V + C * LD;
    uint16_t* Ph = (DG ? X : V) + C * LD;
    uint16_t* Pl = Ph + C * LDP;
    float* bs = reinterpret_cast<float*>(SUMMARY ? V + C * LD : Pl + C * LDP);  // beta[64], then b_C
    float* wo = bs + C + 4;                                                      // e^{b_C - beta}[64]
    float* red = wo + C + 4;                                                     // DG: [4 waves][2][64]
    uint16_t* stage = Q;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, n = lane & 31, half = lane >> 5;
    const SeqWalk walk = seq_walk(d, seq);
    const int nsq = (walk.n + a.m - 1) / a.m;  // segments of this sequence
    const int kbeg = seg * a.m, kend = min(walk.n, kbeg + a.m), cnt = kend - kbeg;
    const bool empty_seq = walk.n == 0 && seg == 0;  // packed input: the state passes through
    if (SUMMARY) {
        // only segments whose end state another segment starts from
        if (cnt <= 0 || (REV ? seg == 0 : seg >= nsq - 1)) return;
    } else if (cnt <= 0 && !empty_seq) {
        return;
    }
    const bool last = empty_seq || (REV ? seg == 0 : seg == nsq - 1);  // this walk ends the sequence

    // state block ib of this wave: S[ib][4g+j] = state[key feature 32 ib + 8g + 4 half + j][value feature 32 wave + n]
    f32x16 S[4];
    _Pragma("unroll") for (int ib = 0; ib < 4; ++ib) S[ib] = f32x16{0};
    if (!SUMMARY) {
        const float* ein = a.nseg > 1 ? a.bound + (size_t(seq) * a.nseg + seg) * D * D
                                      : (a.edge_in ? a.edge_in + size_t(seq) * D * D : nullptr);
        if (ein) {
            _Pragma("unroll") for (int ib = 0; ib < 4; ++ib)
                _Pragma("unroll") for (int x = 0; x < 16; ++x) {
                    const int mm = 32 * ib + 8 * (x >> 2) + 4 * half + (x & 3), nn = 32 * wave + n;
                    S[ib][x] = a.transposed ? ein[nn * D + mm] : ein[mm * D + nn];
                }
        }
    }

    TileRegs rq, rk, rv, rx;
    float gval = 0.f, gtot = 0.f;
    ChunkPos cp{};
    auto chunk_of = [&](int kk) { return REV ? kend - 1 - kk : kbeg + kk; };
    auto gload = [&](int kk) {
        const ChunkPos p = walk_pos(d, walk, chunk_of(min(kk, cnt - 1)));
        if (DEC) {
            const int row = min(lane, p.L - 1), tok = REV ? p.L - 1 - row : row;
            gval = a.g[d.kind == 1 ? size_t(walk.bh % d.H) : p.tok0 + size_t(tok) * p.ts];
        }
        if (!SUMMARY) walk_gload<REV>(rq, a.xq, p.tok0, p.ts, p.L, tid);
        walk_gload<REV>(rk, a.xk, p.tok0, p.ts, p.L, tid);
        walk_gload<REV>(rv, a.xv, p.tok0, p.ts, p.L, tid);
        if (DG) walk_gload<REV>(rx, a.xx, p.tok0, p.ts, p.L, tid);
    };
    if (cnt > 0) gload(0);

    for (int kk = 0; kk < cnt; ++kk) {
        cp = walk_pos(d, walk, chunk_of(kk));
        const int L = cp.L;
        // ---- registers of this chunk -> LDS; decay tables; loads of the next chunk
        if (!SUMMARY) tile_commit(Q, rq, L, tid);
        tile_commit(K, rk, L, tid);
        tile_commit(V, rv, L, tid);
        if (DG) tile_commit(X, rx, L, tid);
        if (DEC) {
            if (wave == 0) {
                const float x = lane < L ? gval : 0.f;
                float inc = x;
                for (int off = 1; off < 64; off <<= 1) {
                    const float y = __shfl_up(inc, off, 64);
                    if (lane >= off) inc += y;
                }
                const float bC = __shfl(inc, 63, 64), beta = REV ? inc - x : inc;
                bs[lane] = beta;
                wo[lane] = __expf(bC - beta);
                if (lane == 0) bs[C] = bC;
                gtot += bC;
            }
        }
        gload(kk + 1);
        __syncthreads();  // (A) tiles and decay tables of this chunk are in LDS
        const float bC = DEC ? bs[C] : 0.f;

        f32x16 O[2];
        float isp[2] = {0.f, 0.f};
        if (!SUMMARY) {
            // ---- inter: O^T[v][j] = e^{beta_j} sum_i S[i][v] q_j[i], the state blocks as A operands straight
            // from the accumulators (head + remainder), the query rows read in the matching k order
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
                    _Pragma("unroll") for (int jb = 0; jb < 2; ++jb) {
                        const bf16x8 qf = frag_perm(Q, LD, 32 * jb + n, 32 * ib + 16 * p, half);
                        O[jb] = mfma(sh, qf, O[jb]);
                        O[jb] = mfma(sl, qf, O[jb]);
                    }
                }
            _Pragma("unroll") for (int jb = 0; jb < 2; ++jb) {
                if (DEC) {
                    const float w = __expf(bs[32 * jb + n]);
                    _Pragma("unroll") for (int x = 0; x < 16; ++x) O[jb][x] *= w;
                }
                if (DG) isp[jb] = row_dot(X, 32 * jb + n, wave, half, O[jb]);
            }
            // ---- scores: each of the three 32 x 32 blocks on or below the diagonal by one wave
            const int pjb = wave ? 1 : 0, prb = wave == 2 ? 1 : 0;  // wave 0: (0,0), wave 1: (1,0), wave 2: (1,1)
            if (wave < 3) {
                f32x16 P = score_block(K, 32 * prb, Q, 32 * pjb, n, half);  // D[m = r][n = j] = k_r . q_j
                walk_mask<DEC>(P, 32 * prb, 32 * pjb + n, bs, half);
                store_block_t_split(Ph, Pl, LDP, 32 * pjb + n, 32 * prb, half, P);
            }
            __syncthreads();  // (C) scores are in LDS; nobody reads Q any more
            // ---- intra: O^T[v][j] += sum_{r <= j} V^T[v][r] P[j][r]
            float pdp[2] = {0.f, 0.f};
            _Pragma("unroll") for (int jb = 0; jb < 2; ++jb) {
                const int j = 32 * jb + n;
                _Pragma("unroll") for (int ks = 0; ks < 2 * (jb + 1); ++ks) {  // keys r >= 32 never reach queries j < 32
                    const bf16x8 vt = frag_tr(V, LD, 16 * ks, 32 * wave, lane);
                    O[jb] = mfma(vt, frag(Ph, LDP, j, 16 * ks + 8 * half), O[jb]);
                    O[jb] = mfma(vt, frag(Pl, LDP, j, 16 * ks + 8 * half), O[jb]);
                }
                if (DG) pdp[jb] = row_dot(X, j, wave, half, O[jb]);
                store_packed(stage, LD, j, 32 * wave, half, pack_block(O[jb]));
            }
            if (DG) {
                _Pragma("unroll") for (int jb = 0; jb < 2; ++jb) {
                    const float pd = pdp[jb] + __shfl_xor(pdp[jb], 32, 64), is = isp[jb] + __shfl_xor(isp[jb], 32, 64);
                    if (half == 0) {
                        red[(wave * 2 + 0) * C + 32 * jb + n] = pd;
                        red[(wave * 2 + 1) * C + 32 * jb + n] = is;
                    }
                }
            }
        }
        // ---- state: S[i][v] = e^{b_C} S[i][v] + sum_t K^T[i][t] (e^{b_C - beta_t} V[t][v]); the weighted value
        // slice of this wave is split into head + remainder in registers
        if (DEC) {
            const float lam = __expf(bC);
            _Pragma("unroll") for (int ib = 0; ib < 4; ++ib)
                _Pragma("unroll") for (int x = 0; x < 16; ++x) S[ib][x] *= lam;
        }
        _Pragma("unroll") for (int ks = 0; ks < 4; ++ks) {
            const u32x4 raw = __builtin_bit_cast(u32x4, frag_tr(V, LD, 16 * ks, 32 * wave, lane));
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
            _Pragma("unroll") for (int ib = 0; ib < 4; ++ib) {
                const bf16x8 ka = frag_tr(K, LD, 16 * ks, 32 * ib, lane);
                S[ib] = mfma(ka, vh, S[ib]);
                if (DEC) S[ib] = mfma(ka, vl, S[ib]);
            }
        }
        __syncthreads();  // (D) the output stage is complete and every read of this chunk's tiles is done
        if (!SUMMARY) {
            // every thread reads back exactly the stage pieces that its own next tile_commit overwrites: no barrier
            walk_store<REV>(a.out, stage, cp.tok0, cp.ts, L, tid);
            if (DG && tid < 64) {
                float pd = 0.f, is = 0.f;
                _Pragma("unroll") for (int wv = 0; wv < 4; ++wv) {
                    pd += red[(wv * 2 + 0) * C + tid];
                    is += red[(wv * 2 + 1) * C + tid];
                }
                if (tid < L) a.pdot[cp.wtok0 + (REV ? L - 1 - tid : tid)] = pd;
                for (int off = 32; off > 0; off >>= 1) is += __shfl_xor(is, off, 64);
                if (tid == 0) a.isum[cp.slot] = is;
            }
        }
    }

    // ---- the state this walk ends with
    if (SUMMARY) {
        float* e = a.bound + (size_t(seq) * a.nseg + (REV ? seg - 1 : seg + 1)) * D * D;
        _Pragma("unroll") for (int ib = 0; ib < 4; ++ib)
            _Pragma("unroll") for (int x = 0; x < 16; ++x)
                e[(32 * ib + 8 * (x >> 2) + 4 * half + (x & 3)) * D + 32 * wave + n] = S[ib][x];
        if (tid == 0) a.gseg[size_t(seq) * a.nseg + seg] = gtot;
        return;
    }
    if (last && a.edge_out) {
        float* e = a.edge_out + size_t(seq) * D * D;
        _Pragma("unroll") for (int ib = 0; ib < 4; ++ib)
            _Pragma("unroll") for (int x = 0; x < 16; ++x) {
                const int mm = 32 * ib + 8 * (x >> 2) + 4 * half + (x & 3), nn = 32 * wave + n;
                e[a.transposed ? nn * D + mm : mm * D + nn] = S[ib][x];
            }
    }
    if (last && a.y0) {
        float z = 0.f;
        if (a.dot_with) {
            const float* w = a.dot_with + size_t(seq) * D * D;
            _Pragma("unroll") for (int ib = 0; ib < 4; ++ib)
                _Pragma("unroll") for (int x = 0; x < 16; ++x) {
                    const int mm = 32 * ib + 8 * (x >> 2) + 4 * half + (x & 3), nn = 32 * wave + n;
                    z += S[ib][x] * w[a.transposed ? nn * D + mm : mm * D + nn];
                }
        }
        for (int off = 32; off > 0; off >>= 1) z += __shfl_xor(z, off, 64);
        __syncthreads();  // the decay tables of the last chunk have been read by everyone
        if (lane == 0) wo[wave] = z;
        __syncthreads();
        if (tid == 0) a.y0[seq] = (wo[0] + wo[1]) + (wo[2] + wo[3]);
    }
}

// forward walker, or the summary pass of either direction
template <bool REV, bool DEC, bool SUMMARY>
__global__ __launch_bounds__(kThreads, 2) void mk_walk(Dims d, WalkArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    walk_body<REV, DEC, false, SUMMARY>(d, a, blockIdx.y, blockIdx.x, smem);
}

// The three walkers of the backward pass in one grid: role 0 = dq (forward in time), 1 = dk, 2 = dv
// (backward in time).  Workgroups are dealt to the 8 XCDs round-robin by linear id; the id is decoded
// so that the three roles of one segment run on one XCD at about the same time (dk and dv read the
// same tiles in the same order and share them in that XCD's L2).
struct WalkTriple { WalkArgs w[3]; };
template <bool DEC, bool DG>
__global__ __launch_bounds__(kThreads, DG ? 1 : 2) void mk_walk_bwd(Dims d, WalkTriple t, int units) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int id = blockIdx.x, full = (units / 8) * 8;
    int role, unit;
    if (id < 3 * full) {
        const int xcd = id & 7, slot = id >> 3;
        role = slot % 3;
        unit = xcd + 8 * (slot / 3);
    } else {  // tail when the number of segments is not a multiple of 8
        role = (id - 3 * full) % 3;
        unit = full + (id - 3 * full) / 3;
    }
    const int nseg = t.w[0].nseg, seq = unit / nseg, seg = unit % nseg;
    if (role == 0) walk_body<false, DEC, DG, false>(d, t.w[0], seq, seg, smem);
    else if (role == 1) walk_body<true, DEC, DG, false>(d, t.w[1], seq, seg, smem);
    else walk_body<true, DEC, false, false>(d, t.w[2], seq, seg, smem);
}

// Entry state of every segment from the segments' own contributions (left by the summary pass in the
// slot of the segment that follows in walk order) and total log-decays: E' = e^{G} E + U, in walk order.
// grid: (128 * 128 / 256, seqs)
template <bool REV>
__global__ __launch_bounds__(kThreads) void mk_bound_scan(Dims d, const float* __restrict__ edge_in, float* __restrict__ bound,
                                                          const float* __restrict__ gseg, int m, int nseg) {
    const int seq = blockIdx.y, e = blockIdx.x * kThreads + threadIdx.x;
    const SeqWalk walk = seq_walk(d, seq);
    const int nsq = max(1, (walk.n + m - 1) / m);
    float* b = bound + size_t(seq) * nseg * D * D + e;
    const float* gs = gseg + size_t(seq) * nseg;
    float E = edge_in ? edge_in[size_t(seq) * D * D + e] : 0.f;
    if (!REV) {
        b[0] = E;
        for (int s = 0; s + 1 < nsq; ++s) {
            E = __expf(gs[s]) * E + b[size_t(s + 1) * D * D];
            b[size_t(s + 1) * D * D] = E;
        }
    } else {
        b[size_t(nsq - 1) * D * D] = E;
        for (int s = nsq - 1; s > 0; --s) {
            E = __expf(gs[s]) * E + b[size_t(s - 1) * D * D];
            b[size_t(s - 1) * D * D] = E;
        }
    }
}

// y_{c+1} = y_0 + sum_{c' <= c} (b_c' - a_c') for the chunks of one sequence, in a fixed order (grid: seqs)
__global__ __launch_bounds__(kThreads) void mk_dg_chunks(Dims d, const float* __restrict__ asum, const float* __restrict__ bsum,
                                                         const float* __restrict__ y0, float* __restrict__ ych) {
    __shared__ float part[kThreads];
    const int seq = blockIdx.x, tid = threadIdx.x;
    const SeqWalk walk = seq_walk(d, seq);
    const size_t base = size_t(walk.bh) * d.N + walk.c0;
    float carry = y0[seq];
    for (int c0 = 0; c0 < walk.n; c0 += kThreads) {
        const int c = c0 + tid;
        float x = c < walk.n ? bsum[base + c] - asum[base + c] : 0.f;
        // inclusive scan over the block: within waves by shuffles, across waves through LDS
        for (int off = 1; off < 64; off <<= 1) {
            const float y = __shfl_up(x, off, 64);
            if ((tid & 63) >= off) x += y;
        }
        if ((tid & 63) == 63) part[tid >> 6] = x;
        __syncthreads();
        float pre = carry;
        for (int w = 0; w < (tid >> 6); ++w) pre += part[w];
        const float tot = ((part[0] + part[1]) + part[2]) + part[3];
        if (c < walk.n) ych[base + c] = pre + x;
        carry += tot;
        __syncthreads();
    }
}

// dg_t = sum_{u >= t, u in chunk} (q_u . dq_u - k_u . dk_u) + y_{c+1}   (grid: N x BH, one wave)
__global__ __launch_bounds__(64) void mk_dg_tokens(Dims d, const float* __restrict__ pf, const float* __restrict__ pr,
                                                   const float* __restrict__ ych, float* __restrict__ dg) {
    const int c = blockIdx.x, bh = blockIdx.y, lane = threadIdx.x;
    const ChunkPos cp = chunk_pos(d, c, bh);
    const int L = cp.L;
    if (L <= 0) return;
    float sfx = lane < L ? pf[cp.wtok0 + lane] - pr[cp.wtok0 + lane] : 0.f;
    for (int off = 1; off < 64; off <<= 1) {
        const float y = __shfl_down(sfx, off, 64);
        if (lane + off < 64) sfx += y;
    }
    float v = lane < L ? sfx + ych[cp.slot] : 0.f;
    if (d.kind == 1) {  // one decay per head: this chunk's share of the sum over tokens
        for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
        if (lane == 0) dg[cp.slot] = v;
    } else if (lane < L) {
        dg[cp.tok0 + size_t(lane) * cp.ts] = v;
    }
}
