// Device helpers shared by the MFMA kernel files: vector types, the 32x32x16 bf16 MFMA and the
// operand access patterns built on its register layout (wave64, l = lane, half = l/32):
//   A operand: lane holds A[m = l%32][k = 8*half + e],  e = 0..7
//   B operand: lane holds B[k = 8*half + e][n = l%32]
//   D result : lane holds D[m = 8*g + 4*half + j][n = l%32] in register 4*g + j
#pragma once
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
// Token-major operand straight out of a row-major [token][feature] LDS tile with the LDS transpose
// read: lane l receives feature col0 + l%32 of tokens row0 + 8*(l/32) + 0..7 (natural k order).
// Each group of 16 lanes reads a 4-token x 16-feature patch as 8-byte pieces (lane r of the group:
// token r/4, features 4*(r%4)..+3) and the hardware hands lane i of the group feature i, 4 tokens.
typedef short s16x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ bf16x8 frag_tr(const uint16_t* tile, int ld, int row0, int col0, int lane) {
    const int r = lane & 15, nblk = (lane >> 4) & 1, half = lane >> 5;
    const uint16_t* p = tile + (row0 + 8 * half + (r >> 2)) * ld + col0 + 16 * nblk + 4 * (r & 3);
    typedef s16x4 __attribute__((address_space(3))) * lds_ptr;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p + 4 * ld));
    u32x2 l2 = __builtin_bit_cast(u32x2, lo), h2 = __builtin_bit_cast(u32x2, hi);
    u32x4 v = {l2.x, l2.y, h2.x, h2.y};
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

// The remainder plane of a chunk state only has to restore a few more bits of the bf16 head (it enters
// one term of the decay gradient), so it is kept as 8-bit floats (1-5-2), scaled by 2^8 to stay clear
// of their underflow: x = head + 2^-8 * rem8 to about 2^-12 relative, in three bytes per element.
constexpr float kRem8Scale = 256.f, kRem8Unscale = 1.f / 256.f;
typedef float f32x2v __attribute__((ext_vector_type(2)));
// 8 such bytes -> bf16 operand (exact: the 8-bit values have two mantissa bits); still scaled by 2^8
__device__ __forceinline__ bf16x8 rem8_to_bf16(u32x2 raw) {
    u32x4 v;
    _Pragma("unroll") for (int p = 0; p < 2; ++p) {
        const f32x2v a = __builtin_amdgcn_cvt_pk_f32_bf8(int(raw[p]), false), b = __builtin_amdgcn_cvt_pk_f32_bf8(int(raw[p]), true);
        v[2 * p] = pack2(a.x, a.y);
        v[2 * p + 1] = pack2(b.x, b.y);
    }
    return __builtin_bit_cast(bf16x8, v);
}

// 64 x 128 bf16 tile: global rows [tok0, tok0+L) -> LDS (row stride LD), rows >= L zero
// (tok0 = row of the first token in src, ts = rows between consecutive tokens)
__device__ __forceinline__ void load_tile(uint16_t* dst, const uint16_t* src, size_t tok0, int ts, int L, int tid) {
    _Pragma("unroll") for (int it = 0; it < 4; ++it) {
        const int p = tid + kThreads * it, row = p >> 4, cp = p & 15;
        // uniform base (scalar registers) + a 32-bit byte offset per lane
        const uint32_t off = (uint32_t(min(row, L - 1)) * uint32_t(ts) * D + cp * 8) * 2;
        const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(reinterpret_cast<const char*>(src + tok0 * D) + off));
        const uint32_t keep = row < L ? 0xffffffffu : 0u;  // branch-free: a branch around a load drains the load queue
        *reinterpret_cast<u32x4*>(dst + row * LD + cp * 8) = u32x4{v.x & keep, v.y & keep, v.z & keep, v.w & keep};
    }
}
// the same in two steps: global -> registers (no operation on the loaded values), registers -> LDS
struct TileRegs { u32x4 v[4]; };
__device__ __forceinline__ void tile_gload(TileRegs& r, const uint16_t* src, size_t tok0, int ts, int L, int tid) {
    _Pragma("unroll") for (int it = 0; it < 4; ++it) {
        const int p = tid + kThreads * it, row = p >> 4, cp = p & 15;
        const uint32_t off = (uint32_t(min(row, L - 1)) * uint32_t(ts) * D + cp * 8) * 2;
        r.v[it] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(reinterpret_cast<const char*>(src + tok0 * D) + off));
    }
}
__device__ __forceinline__ void tile_commit(uint16_t* dst, const TileRegs& r, int L, int tid) {
    _Pragma("unroll") for (int it = 0; it < 4; ++it) {
        const int p = tid + kThreads * it, row = p >> 4, cp = p & 15;
        const uint32_t keep = row < L ? 0xffffffffu : 0u;
        *reinterpret_cast<u32x4*>(dst + row * LD + cp * 8) = u32x4{r.v[it].x & keep, r.v[it].y & keep, r.v[it].z & keep, r.v[it].w & keep};
    }
}
// LDS tile (row stride LD) rows [0, L) -> global
__device__ __forceinline__ void store_tile(uint16_t* dst, const uint16_t* src, size_t tok0, int ts, int L, int tid) {
    _Pragma("unroll") for (int it = 0; it < 4; ++it) {
        const int p = tid + kThreads * it, row = p >> 4, cp = p & 15;
        const uint32_t off = (uint32_t(row) * uint32_t(ts) * D + cp * 8) * 2;
        if (row < L)
            __builtin_nontemporal_store(*reinterpret_cast<const u32x4*>(src + row * LD + cp * 8),
                                        reinterpret_cast<u32x4*>(reinterpret_cast<char*>(dst + tok0 * D) + off));
    }
}

struct PackedBlock { u32x2 v[4]; };  // a D-layout block rounded to bf16: v[g] = rows 8g + 4half + 0..3
__device__ __forceinline__ PackedBlock pack_block(const f32x16& d) {
    PackedBlock p;
    _Pragma("unroll") for (int g = 0; g < 4; ++g)
        p.v[g] = u32x2{pack2(d[4 * g + 0], d[4 * g + 1]), pack2(d[4 * g + 2], d[4 * g + 3])};
    return p;
}
__device__ __forceinline__ void store_packed(uint16_t* dst, int ld, int nrow, int m0, int half, const PackedBlock& p) {
    _Pragma("unroll") for (int g = 0; g < 4; ++g)
        *reinterpret_cast<u32x2*>(dst + nrow * ld + m0 + 8 * g + 4 * half) = p.v[g];
}

}  // namespace
}  // namespace lsm
