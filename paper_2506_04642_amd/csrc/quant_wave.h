// Device helpers of the quantiser that more than one translation unit uses: the 16-bit
// conversions, the group metadata and code arithmetic of arxiv 2506.04642's deviation quantiser
// (Sec. 3.2 Eq. 3-4 with asymmetric min/max groups; the S and M of Algorithm 1), and the
// one-wavefront-per-item lane layout (lane l owns tokens 8 (l & 3) .. + 7 of channels
// 8 (l >> 2) .. + 7 of a 32-token x 128-channel item) with its lane exchanges and word packers.
// Every translation unit that includes this file is compiled with -ffp-contract=off: each
// binary32 operation rounds once, in the order written.
#pragma once
#include "tadakv_internal.h"
#include <hip/hip_fp16.h>
#include <type_traits>

namespace tadakv {
namespace {

__device__ __forceinline__ float widen16(uint16_t v, int dtype)
{
    if (dtype == 1) return __uint_as_float((uint32_t)v << 16); // bfloat16
    return __half2float(__ushort_as_half(v));
}

__device__ __forceinline__ uint16_t f16_rne(float f) { return __half_as_ushort(__float2half_rn(f)); }
__device__ __forceinline__ float f16_val(uint16_t h) { return __half2float(__ushort_as_half(h)); }

// binary32 -> the cache's 16-bit type, round to nearest even
__device__ __forceinline__ uint16_t narrow16(float f, int dtype)
{
    if (dtype == 1) {
        const uint32_t u = __float_as_uint(f);
        if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x0040u);
        return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
    }
    return f16_rne(f);
}

// f rounded to the 16-bit type (DT: 0 binary16, 1 bfloat16) and widened again, without branches
template <int DT> __device__ __forceinline__ float round16(float f)
{
    if (DT == 1) return (float)(__bf16)f; // the conversion instruction of this chip: round to nearest, ties to even
    return __half2float(__float2half_rn(f));
}

// Two values that the 16-bit type holds exactly (DT: 0 binary16, 1 bfloat16), as the type's bit patterns
// in one word, a in the low half: one instruction.
template <int DT> __device__ __forceinline__ uint32_t pack16_exact(float a, float b)
{
    if (DT == 1) return __builtin_amdgcn_perm(__float_as_uint(b), __float_as_uint(a), 0x07060302u);
    typedef _Float16 h2_t __attribute__((ext_vector_type(2)));
    return __builtin_bit_cast(uint32_t, (h2_t)__builtin_amdgcn_cvt_pkrtz(a, b)); // (exact values: no rounding takes place)
}

// One rotated pair: (a, b) -> (a cos - b sin, b cos + a sin), rounded to the 16-bit type and widened again.
template <int DT>
__device__ __forceinline__ void rope_pair_t(float xa, float xb, float c, float s, float &ya, float &yb)
{
    const float p1 = xa * c, p2 = xb * s, p3 = xb * c, p4 = xa * s;
    ya = round16<DT>(p1 - p2);
    yb = round16<DT>(p3 + p4);
}
__device__ __forceinline__ void rope_pair(float xa, float xb, float c, float s, int dtype, float &ya, float &yb)
{
    if (dtype == 1) rope_pair_t<1>(xa, xb, c, s, ya, yb);
    else rope_pair_t<0>(xa, xb, c, s, ya, yb);
}

// Channel c of a new key row after the rotation (row: the 128 raw elements, cs / sn: the token's 64 angles).
__device__ __forceinline__ float rope_elem(const uint16_t *row, int c, const float *cs, const float *sn, int mode, int dtype)
{
    const int i = mode == 1 ? (c & 63) : (c >> 1);
    const int ia = mode == 1 ? i : 2 * i, ib = mode == 1 ? i + 64 : 2 * i + 1;
    float ya, yb;
    rope_pair(widen16(row[ia], dtype), widen16(row[ib], dtype), cs[i], sn[i], dtype, ya, yb);
    return c == ia ? ya : yb;
}

// largest binary16 <= f
__device__ __forceinline__ uint16_t f16_down(float f)
{
    uint16_t h = f16_rne(f);
    if (f16_val(h) > f) {
        if ((h & 0x7FFFu) == 0) h = 0x8001u;
        else h = (h & 0x8000u) ? (uint16_t)(h + 1) : (uint16_t)(h - 1);
    }
    return h;
}
// smallest binary16 >= f
__device__ __forceinline__ uint16_t f16_up(float f)
{
    uint16_t h = f16_rne(f);
    if (f16_val(h) < f) {
        if ((h & 0x7FFFu) == 0) h = 0x0001u;
        else h = (h & 0x8000u) ? (uint16_t)(h - 1) : (uint16_t)(h + 1);
    }
    return h;
}

__device__ __forceinline__ void group_meta(float mn, float mx, int qmax, uint16_t &s16, uint16_t &z16,
                                           float &s, float &z)
{
    if (mn == 0.0f) mn = 0.0f; // -0 -> +0
    if (mx == 0.0f) mx = 0.0f;
    z16 = f16_down(mn);
    z = f16_val(z16);
    float rng = mx - z;
    float s32 = rng / (float)qmax;
    s16 = f16_up(s32);
    s = f16_val(s16);
}

// code = clamp(rint((dev - z) / s), 0, qmax).  The quotient is formed with the group's
// reciprocal r = 1/s (one IEEE division per group) and one fused correction step:
//   q = x r;  e = fma(-q, s, x);  q' = fma(e, r, q)
// which equals the correctly rounded x / s whenever r is the correctly rounded reciprocal and
// the significand of s is not all ones (Markstein's division theorem); s is a binary16 value,
// so its binary32 significand has at most 11 leading bits set.
__device__ __forceinline__ uint32_t quant_code(float dev, float s, float rs, float z, float qmaxf)
{
    // A constant group has s == 0 and is given rs == 0: then dev == z, every term below is zero
    // and the code is 0 without a special case.  0 <= u < qmax + 1/2 by construction of z and s
    // (z <= dev; scale rounded up), so the clamp never binds.  Rounding to the nearest integer,
    // ties to even, is the addition of 2^23 (the sum's unit in the last place is 1); the integer is
    // then the sum's significand field, of which the code's bits are kept.
    const float xv = dev - z;
    const float q = xv * rs;
    const float e = __builtin_fmaf(-q, s, xv);
    const float u = __builtin_fmaf(e, rs, q);
    return __float_as_uint(u + 0x1p23f) & (uint32_t)qmaxf;
}

// The quotient alone (see quant_code), and four of them rounded to the nearest integer (ties to
// even), clamped to 0 .. 255 and packed as the bytes of a word by the conversion instruction that
// does all three at once.
__device__ __forceinline__ float quant_quotient(float dev, float s, float rs, float z)
{
    const float xv = dev - z;
    const float q = xv * rs;
    const float e = __builtin_fmaf(-q, s, xv);
    return __builtin_fmaf(e, rs, q);
}
__device__ __forceinline__ uint32_t pack4_u8(float u0, float u1, float u2, float u3)
{
    uint32_t w = __builtin_amdgcn_cvt_pk_u8_f32(u0, 0, 0);
    w = __builtin_amdgcn_cvt_pk_u8_f32(u1, 1, w);
    w = __builtin_amdgcn_cvt_pk_u8_f32(u2, 2, w);
    return __builtin_amdgcn_cvt_pk_u8_f32(u3, 3, w);
}

template <int CTRL> __device__ __forceinline__ uint32_t dpp_u(uint32_t x)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, 0xF, 0xF, true);
}
template <int CTRL> __device__ __forceinline__ float dpp_f(float x) { return __uint_as_float(dpp_u<CTRL>(__float_as_uint(x))); }
// value of quad lane P in every lane of the quad
template <int P> __device__ __forceinline__ uint32_t quad_bcast_u(uint32_t x) { return dpp_u<P * 0x55>(x); }
template <int P> __device__ __forceinline__ float quad_bcast_f(float x) { return dpp_f<P * 0x55>(x); }
// value of lane src (any lane), through the LDS crossbar
__device__ __forceinline__ uint32_t from_lane_u(uint32_t x, int src) { return (uint32_t)__builtin_amdgcn_ds_bpermute(src << 2, (int)x); }
__device__ __forceinline__ float from_lane_f(float x, int src) { return __uint_as_float(from_lane_u(__float_as_uint(x), src)); }
// one of four by a lane-dependent index 0..3
template <class T> __device__ __forceinline__ T pick4(int i, T a0, T a1, T a2, T a3)
{
    const T lo = i & 1 ? a1 : a0, hi = i & 1 ? a3 : a2;
    return i & 2 ? hi : lo;
}

struct MetaOut {
    uint32_t pk; // scale | zero << 16, binary16 patterns
    float rs;    // correctly rounded 1 / scale, 0 for a constant group
};
__device__ __forceinline__ MetaOut meta_of(float mn, float mx, int qmax)
{
    uint16_t s16, z16;
    float sc, z;
    group_meta(mn, mx, qmax, s16, z16, sc, z);
    MetaOut o;
    o.pk = (uint32_t)s16 | ((uint32_t)z16 << 16);
    o.rs = sc != 0.0f ? 1.0f / sc : 0.0f;
    return o;
}

// Rotation of this lane's 8 x 8 key values, token pair by token pair (Alg. 1 step 5).  With the
// (i, i + 64) pairing the partner channel lives in lane l ^ 32 (same tokens); with (2i, 2i + 1)
// it is the neighbouring register.  Rows that come from the residual buffer (tn < 0) were
// rotated when they were stored.
template <int DT>
__device__ __forceinline__ void rope_in_lanes(float (&x)[8][8], const AppendArgs &a, int tn0, int lane)
{
    const int c8 = lane >> 2;
    const bool half_mode = a.rope == 1;
    // first of this lane's pair indices: 8 pairs (half) or 4 pairs (interleaved)
    const int i0 = half_mode ? 8 * (c8 & 7) : 4 * c8;
#pragma unroll
    for (int jb = 0; jb < 8; jb += 2) {
        float4 cs[2][2], sn[2][2];
#pragma unroll
        for (int d = 0; d < 2; d++) {
            int tn = tn0 + jb + d;
            tn = tn < 0 ? 0 : tn;
            const float *pc = a.rope_cos + (long long)tn * 64 + i0, *ps = a.rope_sin + (long long)tn * 64 + i0;
            cs[d][0] = *(const float4 *)pc;
            sn[d][0] = *(const float4 *)ps;
            if (half_mode) {
                cs[d][1] = *(const float4 *)(pc + 4);
                sn[d][1] = *(const float4 *)(ps + 4);
            } else {
                cs[d][1] = float4{0.0f, 0.0f, 0.0f, 0.0f};
                sn[d][1] = float4{0.0f, 0.0f, 0.0f, 0.0f};
            }
        }
#pragma unroll
        for (int d = 0; d < 2; d++) {
            const int j = jb + d;
            const bool turn = tn0 + j >= 0;
            const float cv[8] = {cs[d][0].x, cs[d][0].y, cs[d][0].z, cs[d][0].w, cs[d][1].x, cs[d][1].y, cs[d][1].z, cs[d][1].w};
            const float sv[8] = {sn[d][0].x, sn[d][0].y, sn[d][0].z, sn[d][0].w, sn[d][1].x, sn[d][1].y, sn[d][1].z, sn[d][1].w};
            if (half_mode) {
                // lower channel of the pair: x cos - partner sin; upper: x cos + partner sin.  The sign
                // goes into the sine once per token (a product with the negated sine is the negated
                // product, and adding that is the subtraction, bit for bit).
                const bool lower = c8 < 8;
#pragma unroll
                for (int e = 0; e < 8; e++) {
                    const float sg = lower ? -sv[e] : sv[e];
                    const float xp = from_lane_f(x[j][e], lane ^ 32);
                    const float p1 = x[j][e] * cv[e], p2 = xp * sg;
                    const float y = round16<DT>(p1 + p2);
                    x[j][e] = turn ? y : x[j][e];
                }
            } else {
#pragma unroll
                for (int k = 0; k < 4; k++) {
                    const float xa = x[j][2 * k], xb = x[j][2 * k + 1];
                    float ya, yb;
                    rope_pair_t<DT>(xa, xb, cv[k], sv[k], ya, yb);
                    x[j][2 * k] = turn ? ya : xa;
                    x[j][2 * k + 1] = turn ? yb : xb;
                }
            }
        }
    }
}

// Minimum / maximum as the bare instructions.  fminf / fmaxf make the compiler put a quieting
// instruction in front of every operand it cannot prove to be free of signalling NaNs (every value
// that came through a lane exchange, for one), which doubled the cost of the extrema below; the
// instructions themselves return the other operand when one is a NaN, like fminf / fmaxf.
__device__ __forceinline__ float vmin(float a, float b) { float r; asm("v_min_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b)); return r; }
__device__ __forceinline__ float vmax(float a, float b) { float r; asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b)); return r; }
__device__ __forceinline__ float vmin3(float a, float b, float c) { float r; asm("v_min3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c)); return r; }
__device__ __forceinline__ float vmax3(float a, float b, float c) { float r; asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c)); return r; }

// The eight 16-byte pieces a lane loaded (eight 16-bit values each), widened to binary32; the
// branch on the input type is taken once for all 64 values instead of as a select per value.
__device__ __forceinline__ void widen_pieces(const uint4 (&pre)[8], int dtype, float (&x)[8][8])
{
    if (dtype == 1) {
#pragma unroll
        for (int j = 0; j < 8; j++) {
            const uint32_t wv[4] = {pre[j].x, pre[j].y, pre[j].z, pre[j].w};
#pragma unroll
            for (int k = 0; k < 4; k++) {
                x[j][2 * k] = __uint_as_float(wv[k] << 16);
                x[j][2 * k + 1] = __uint_as_float(wv[k] & 0xFFFF0000u);
            }
        }
    } else {
#pragma unroll
        for (int j = 0; j < 8; j++) {
            const uint32_t wv[4] = {pre[j].x, pre[j].y, pre[j].z, pre[j].w};
#pragma unroll
            for (int k = 0; k < 4; k++) {
                x[j][2 * k] = f16_val((uint16_t)(wv[k] & 0xFFFFu));
                x[j][2 * k + 1] = f16_val((uint16_t)(wv[k] >> 16));
            }
        }
    }
}

// Codes and packed words of 32 key tokens held as deviations x[token j][channel e] (lane = (tg, c8)),
// given the per-channel metadata; `half` is the 32-token half of the block (0 for blocks of 32).
// A key word runs along channels.
template <int BITS>
__device__ __forceinline__ void emit_key_words(const float (&x)[8][8], const float (&sc)[8], const float (&rs)[8],
                                               const float (&z)[8], int half, int lane, unsigned char *codes_out)
{
    const int tg = lane & 3, c8 = lane >> 2;
    const int tt = 2 * half + (tg >> 1), jj = c8 >> 2; // 16-token tile of the block, channel-tile pair
#pragma unroll
    for (int j = 0; j < 8; j++) {
        const int n = 8 * (tg & 1) + j;
        float uq[8];
#pragma unroll
        for (int e = 0; e < 8; e++) uq[e] = quant_quotient(x[j][e], sc[e], rs[e], z[e]);
        const uint32_t clo = pack4_u8(uq[0], uq[1], uq[2], uq[3]), chi = pack4_u8(uq[4], uq[5], uq[6], uq[7]);
        if (BITS == 8) {
            const int piece = ((tt * 2 + ((c8 >> 1) & 1)) * 4 + jj) * 16 + n;
            *(uint2 *)(codes_out + (piece * 4 + 2 * (c8 & 1)) * 4) = uint2{clo, chi};
        } else if (BITS == 4) {
            const uint32_t w = clo | (chi << 4); // byte y: codes y and y + 4
            ((uint32_t *)codes_out)[((tt * 4 + jj) * 16 + n) * 4 + (c8 & 3)] = w;
        } else {
            // 16 channels per word: this lane's half, shifted into place, joined with the
            // neighbouring channel octet's (lane ^ 4); two token tiles share a piece
            uint32_t w = clo | (chi << 2); // byte y: codes y and y + 4 in its low four bits
            w <<= 4 * (c8 & 1);
            w |= from_lane_u(w, lane ^ 4);
            if ((j >> 2) == (c8 & 1))
                ((uint32_t *)codes_out)[(((tt >> 1) * 4 + jj) * 16 + n) * 4 + (((tt & 1) << 1) | ((c8 >> 1) & 1))] = w;
        }
    }
}

// Metadata, codes and packed words of 32 value tokens held as deviations x[token j][channel e]:
// one group per (token, GC channels) = eight channels in the lane times GC / 8 lanes.  NT is the
// number of 16-token tiles of the block; meta_out points at the block's (scale, zero) array.
template <int GC, int BITS, int NT>
__device__ __forceinline__ void emit_value_half(const float (&x)[8][8], int half, int lane, unsigned char *codes_out,
                                                unsigned char *meta_out)
{
    constexpr int NGV = kHeadDim / GC;
    constexpr int qmax = (1 << BITS) - 1;
    const int tg = lane & 3, c8 = lane >> 2;
    float mn[8], mx[8];
#pragma unroll
    for (int j = 0; j < 8; j++) {
        float lo = vmin(vmin3(x[j][0], x[j][1], x[j][2]), vmin3(x[j][3], x[j][4], vmin3(x[j][5], x[j][6], x[j][7])));
        float hi = vmax(vmax3(x[j][0], x[j][1], x[j][2]), vmax3(x[j][3], x[j][4], vmax3(x[j][5], x[j][6], x[j][7])));
        // lanes 4 and 8 apart in the row of 16 (rotations: the coset is covered either way)
        lo = vmin(lo, dpp_f<0x124>(lo));
        hi = vmax(hi, dpp_f<0x124>(hi));
        lo = vmin(lo, dpp_f<0x128>(lo));
        hi = vmax(hi, dpp_f<0x128>(hi));
        if (GC >= 64) {
            lo = vmin(lo, from_lane_f(lo, lane ^ 16));
            hi = vmax(hi, from_lane_f(hi, lane ^ 16));
        }
        if (GC >= 128) {
            lo = vmin(lo, from_lane_f(lo, lane ^ 32));
            hi = vmax(hi, from_lane_f(hi, lane ^ 32));
        }
        mn[j] = lo;
        mx[j] = hi;
    }
    // lane with q4 = c8 & 3 works out tokens 2 q4 and 2 q4 + 1 of its group, then the four share
    const int q4 = c8 & 3;
    const MetaOut ma = meta_of(pick4(q4, mn[0], mn[2], mn[4], mn[6]), pick4(q4, mx[0], mx[2], mx[4], mx[6]), qmax);
    const MetaOut mb = meta_of(pick4(q4, mn[1], mn[3], mn[5], mn[7]), pick4(q4, mx[1], mx[3], mx[5], mx[7]), qmax);
    if ((c8 & (GC / 8 - 1)) == q4) {
        const int gam = c8 / (GC / 8), t = 32 * half + 8 * tg + 2 * q4;
        *(uint32_t *)(meta_out + (t * NGV + gam) * 4) = ma.pk;
        *(uint32_t *)(meta_out + ((t + 1) * NGV + gam) * 4) = mb.pk;
    }
    float sc[8], z[8], rs[8];
#pragma unroll
    for (int j = 0; j < 8; j++) {
        const int src = (lane & ~12) | ((j >> 1) << 2);
        const uint32_t pk = from_lane_u((j & 1) ? mb.pk : ma.pk, src);
        rs[j] = from_lane_f((j & 1) ? mb.rs : ma.rs, src);
        sc[j] = f16_val((uint16_t)(pk & 0xFFFFu));
        z[j] = f16_val((uint16_t)(pk >> 16));
    }
    // codes and words: a value word runs along tokens
    const int tt = 2 * half + (tg >> 1);
#pragma unroll
    for (int e = 0; e < 8; e++) {
        const int n = 8 * (c8 & 1) + e;
        float uq[8];
#pragma unroll
        for (int j = 0; j < 8; j++) uq[j] = quant_quotient(x[j][e], sc[j], rs[j], z[j]);
        const uint32_t clo = pack4_u8(uq[0], uq[1], uq[2], uq[3]), chi = pack4_u8(uq[4], uq[5], uq[6], uq[7]);
        if (BITS == 8) {
            const int piece = ((c8 >> 1) * NT + tt) * 16 + n;
            *(uint2 *)(codes_out + (piece * 4 + 2 * (tg & 1)) * 4) = uint2{clo, chi};
        } else if (BITS == 4) {
            const uint32_t w = clo | (chi << 4); // byte y: codes y and y + 4
            const int piece = ((c8 >> 2) * NT + tt) * 16 + n;
            ((uint32_t *)codes_out)[piece * 4 + 2 * ((c8 >> 1) & 1) + (tg & 1)] = w;
        } else {
            uint32_t w = clo | (chi << 2); // byte y: codes y and y + 4 in its low four bits
            w <<= 4 * (tg & 1);
            w |= dpp_u<0xB1>(w);
            const int piece = ((c8 >> 3) * NT + tt) * 16 + n;
            if ((e >> 2) == (tg & 1)) ((uint32_t *)codes_out)[piece * 4 + ((c8 >> 1) & 3)] = w;
        }
    }
}

// Key metadata of the eight channels of a lane from the groups' extrema (equal in the four lanes
// of a quad): quad lane tg works out channels 2 tg and 2 tg + 1, then all share; lane tg == 0
// stores the packed scale / zero rows.
__device__ __forceinline__ void key_metadata(const float (&mn)[8], const float (&mx)[8], int qmax, int lane,
                                             unsigned char *scale_out, unsigned char *zero_out, float (&sc)[8],
                                             float (&rs)[8], float (&z)[8])
{
    const int tg = lane & 3, c8 = lane >> 2;
    const MetaOut ma = meta_of(pick4(tg, mn[0], mn[2], mn[4], mn[6]), pick4(tg, mx[0], mx[2], mx[4], mx[6]), qmax);
    const MetaOut mb = meta_of(pick4(tg, mn[1], mn[3], mn[5], mn[7]), pick4(tg, mx[1], mx[3], mx[5], mx[7]), qmax);
    uint32_t pk[8];
    pk[0] = quad_bcast_u<0>(ma.pk); rs[0] = quad_bcast_f<0>(ma.rs);
    pk[1] = quad_bcast_u<0>(mb.pk); rs[1] = quad_bcast_f<0>(mb.rs);
    pk[2] = quad_bcast_u<1>(ma.pk); rs[2] = quad_bcast_f<1>(ma.rs);
    pk[3] = quad_bcast_u<1>(mb.pk); rs[3] = quad_bcast_f<1>(mb.rs);
    pk[4] = quad_bcast_u<2>(ma.pk); rs[4] = quad_bcast_f<2>(ma.rs);
    pk[5] = quad_bcast_u<2>(mb.pk); rs[5] = quad_bcast_f<2>(mb.rs);
    pk[6] = quad_bcast_u<3>(ma.pk); rs[6] = quad_bcast_f<3>(ma.rs);
    pk[7] = quad_bcast_u<3>(mb.pk); rs[7] = quad_bcast_f<3>(mb.rs);
    if (tg == 0) {
        uint32_t sw[4], zw[4];
#pragma unroll
        for (int k = 0; k < 4; k++) {
            sw[k] = (pk[2 * k] & 0xFFFFu) | (pk[2 * k + 1] << 16);
            zw[k] = (pk[2 * k] >> 16) | (pk[2 * k + 1] & 0xFFFF0000u);
        }
        *(uint4 *)(scale_out + c8 * 16) = uint4{sw[0], sw[1], sw[2], sw[3]};
        *(uint4 *)(zero_out + c8 * 16) = uint4{zw[0], zw[1], zw[2], zw[3]};
    }
#pragma unroll
    for (int e = 0; e < 8; e++) {
        sc[e] = f16_val((uint16_t)(pk[e] & 0xFFFFu));
        z[e] = f16_val((uint16_t)(pk[e] >> 16));
    }
}


} // namespace
} // namespace tadakv
