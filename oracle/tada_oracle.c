/*
 * tada_oracle.c -- TEST INFRASTRUCTURE, not the product.
 *
 * A plain, slow, single-threaded CPU statement of what the TaDA hot path computes
 * (arxiv 2506.04642): mean-centring of key/value activations (Sec. 3.1, Eq. 1-2),
 * deviations (Sec. 3.2, Eq. 3-4), group quantisation of the deviations to nbits with
 * 16-bit scale / zero-point metadata (Sec. 3 memory formula; Algorithm 1's S and M),
 * reconstruction (Eq. 7-8) and softmax attention over the reconstructed cache plus
 * the uncompressed residual tokens (Eq. 5-6, Eq. 9-10); the rotary embedding of the
 * keys that Algorithm 1 (step 5) fuses with their compression; and the value projection
 * that step 3 fuses with the compression of the values.
 *
 * Only tests, the smoke check and the cpu_baseline leg of the benchmark may call this
 * file.  It shares no code, header, table or constant with the HIP path.
 *
 * Encoder arithmetic is IEEE binary32, one rounding per operation, evaluated in the
 * order written (compile with -ffp-contract=off, no fast-math).  Attention is binary64.
 *
 * The paper leaves quantize(), S and M undefined; the reading taken here is asymmetric
 * uniform min/max quantisation per group, keys grouped per channel over a block of
 * tokens and values per token over a group of channels (the KIVI arrangement the paper
 * refers to in Sec. 1 and Sec. 3.3), sign convention D = x - mean, x^ = mean + deq(D).
 *
 * Layout conventions of this file (logical, unpacked):
 *   x      [G][H][d]   16-bit inputs of one batch element, one block of G tokens
 *   codes  [H][G][d]   one byte per code
 *   K meta scale,zero [H][d];  V meta scale,zero [H][G][d/Gc]
 *   mean   CHANNEL_BLOCK: [H][d] (mean over the block's tokens, per head and channel)
 *          CROSS_HEAD   : [G][d] (mean over heads, per token and channel; Eq. 1-2)
 *          NONE         : unused
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORC_F16 = 0, ORC_BF16 = 1 };
enum { ORC_MEAN_CHANNEL_BLOCK = 0, ORC_MEAN_CROSS_HEAD = 1, ORC_MEAN_NONE = 2 };
enum { ORC_K = 0, ORC_V = 1 };

/* ------------------------------------------------------------------ 16-bit formats */

static float bits_to_f32(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }
static uint32_t f32_to_bits(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }

/* IEEE binary16 -> binary32, exact. */
float orc_f16_to_f32(uint16_t h)
{
    uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    uint32_t exp = (h >> 10) & 0x1Fu;
    uint32_t man = h & 0x3FFu;
    if (exp == 0x1Fu) return bits_to_f32(sign | 0x7F800000u | (man << 13));
    if (exp == 0) {
        /* zero or subnormal: value = man * 2^-24 */
        float v = (float)man * 5.9604644775390625e-08f;
        return sign ? -v : v;
    }
    return bits_to_f32(sign | ((exp + 112u) << 23) | (man << 13));
}

/* bfloat16 -> binary32, exact (bf16 is the top half of a binary32). */
float orc_bf16_to_f32(uint16_t b) { return bits_to_f32((uint32_t)b << 16); }

/* binary32 -> binary16, round to nearest, ties to even. */
uint16_t orc_f32_to_f16_rne(float f)
{
    uint32_t u = f32_to_bits(f);
    uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    uint32_t a = u & 0x7FFFFFFFu;
    if (a >= 0x7F800000u) /* inf / nan */
        return (uint16_t)(sign | 0x7C00u | ((a > 0x7F800000u) ? 0x200u : 0u));
    if (a >= 0x477FF000u) /* >= 65520 rounds to infinity */
        return (uint16_t)(sign | 0x7C00u);
    if (a < 0x33000000u) /* below 2^-25 (half the smallest subnormal) rounds to zero */
        return sign;
    int e = (int)(a >> 23) - 127;          /* unbiased exponent */
    uint32_t m = (a & 0x7FFFFFu) | 0x800000u; /* 24-bit significand */
    int shift;                              /* bits dropped from the significand */
    uint32_t base;
    if (e >= -14) { shift = 13; base = (uint32_t)(e + 15) << 10; }
    else          { shift = 13 + (-14 - e); base = 0; }
    uint32_t kept = m >> shift;
    uint32_t rem = m & ((1u << shift) - 1u);
    uint32_t half = 1u << (shift - 1);
    if (rem > half || (rem == half && (kept & 1u))) kept++;
    /* for normals kept holds the hidden bit: adding it to base bumps the exponent
       field by one, so subtract one exponent step first; a carry out of the
       significand then correctly lands in the exponent. */
    uint32_t h = (e >= -14) ? (base - 0x400u + kept) : kept;
    return (uint16_t)(sign | h);
}

/* next binary16 toward -infinity / +infinity of a finite pattern */
static uint16_t f16_step_down(uint16_t h)
{
    if ((h & 0x7FFFu) == 0) return 0x8001u;           /* +-0 -> smallest negative */
    return (h & 0x8000u) ? (uint16_t)(h + 1) : (uint16_t)(h - 1);
}
static uint16_t f16_step_up(uint16_t h)
{
    if ((h & 0x7FFFu) == 0) return 0x0001u;
    return (h & 0x8000u) ? (uint16_t)(h - 1) : (uint16_t)(h + 1);
}

/* largest binary16 <= f  (f finite, |f| < 65504) */
uint16_t orc_f32_to_f16_down(float f)
{
    uint16_t h = orc_f32_to_f16_rne(f);
    if (orc_f16_to_f32(h) > f) h = f16_step_down(h);
    return h;
}
/* smallest binary16 >= f */
uint16_t orc_f32_to_f16_up(float f)
{
    uint16_t h = orc_f32_to_f16_rne(f);
    if (orc_f16_to_f32(h) < f) h = f16_step_up(h);
    return h;
}

static float widen(uint16_t v, int dtype)
{
    return dtype == ORC_BF16 ? orc_bf16_to_f32(v) : orc_f16_to_f32(v);
}

/* binary32 -> bfloat16, round to nearest, ties to even (bfloat16 keeps the top 16 bits). */
uint16_t orc_f32_to_bf16_rne(float f)
{
    uint32_t u = f32_to_bits(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x0040u); /* nan stays nan */
    uint32_t kept = u >> 16, rem = u & 0xFFFFu;
    if (rem > 0x8000u || (rem == 0x8000u && (kept & 1u))) kept++; /* a carry runs into the exponent: correct */
    return (uint16_t)kept;
}

static uint16_t narrow(float f, int dtype)
{
    return dtype == ORC_BF16 ? orc_f32_to_bf16_rne(f) : orc_f32_to_f16_rne(f);
}

/* ------------------------------------------------------------------ rotary embedding */

enum { ORC_ROPE_HALF = 0, ORC_ROPE_INTERLEAVED = 1 };

/*
 * Rotary position embedding of key rows, the step that Algorithm 1 (step 5) fuses with the
 * compression of the keys (Sec. 3.4; App. A).  Pair i of a row, channels (a, b), is turned by the
 * angle the caller's tables give for (token, i):
 *     y_a = x_a cos - x_b sin        y_b = x_b cos + x_a sin
 * with (a, b) = (i, i + d/2) for ORC_ROPE_HALF and (2i, 2i + 1) for ORC_ROPE_INTERLEAVED.
 * binary32: each product is rounded, then the difference / sum, then the result is rounded to
 * the 16-bit type (nearest even) -- the rotated key is a 16-bit tensor, as it is when the
 * rotation runs as a step of its own before the cache update.
 * x, y [T][H][d] 16-bit; cs, sn [T][d/2] binary32.
 */
int orc_rope(const uint16_t *x, int dtype, int T, int H, int d, const float *cs, const float *sn,
             int pairing, uint16_t *y)
{
    if (d % 2 || (pairing != ORC_ROPE_HALF && pairing != ORC_ROPE_INTERLEAVED)) return -1;
    const int hd = d / 2;
    for (int t = 0; t < T; t++)
        for (int h = 0; h < H; h++) {
            const uint16_t *row = x + ((size_t)t * H + h) * d;
            uint16_t *out = y + ((size_t)t * H + h) * d;
            for (int i = 0; i < hd; i++) {
                const int a = pairing == ORC_ROPE_HALF ? i : 2 * i;
                const int b = pairing == ORC_ROPE_HALF ? i + hd : 2 * i + 1;
                const float xa = widen(row[a], dtype), xb = widen(row[b], dtype);
                const float c = cs[(size_t)t * hd + i], s = sn[(size_t)t * hd + i];
                const float p1 = xa * c, p2 = xb * s, p3 = xb * c, p4 = xa * s;
                out[a] = narrow(p1 - p2, dtype);
                out[b] = narrow(p3 + p4, dtype);
            }
        }
    return 0;
}

/* ------------------------------------------------------------------ value projection */

/* binary64 -> the 16-bit type, ONE rounding (nearest, ties to even): the value is scaled by a power
   of two so that the target's unit in the last place becomes 1, rounded to an integer by the
   default rounding mode, and scaled back; what remains is exactly representable in the 16-bit
   type (or overflows to infinity), so the final narrowing through binary32 is exact.  Going
   through binary32 first would round twice. */
uint16_t orc_f64_to_16_rne(double v, int dtype)
{
    if (v != v) return dtype == ORC_BF16 ? 0x7FC0u : 0x7E00u;
    if (v == 0.0 || isinf(v)) return narrow((float)v, dtype);
    const int sig = dtype == ORC_BF16 ? 8 : 11;      /* significand bits, hidden one included */
    const int emin = dtype == ORC_BF16 ? -126 : -14; /* exponent of the smallest normal */
    int e;
    (void)frexp(v, &e); /* |v| in [2^(e-1), 2^e) */
    int ulp_exp = (e - 1) - (sig - 1);
    if (ulp_exp < emin - (sig - 1)) ulp_exp = emin - (sig - 1); /* subnormal range: fixed spacing */
    const double r = ldexp(nearbyint(ldexp(v, -ulp_exp)), ulp_exp);
    return narrow((float)r, dtype); /* exact, or beyond the largest finite value: infinity */
}

/*
 * The value projection of Algorithm 1 step 3 (CompressV(X, W_V): the linear projection whose
 * result is mean-centred and quantised): v[r][o] = sum_k x[r][k] * w[o][k], every product and the
 * sum in binary64 in index order, rounded once to the 16-bit type -- the projected value is a
 * 16-bit tensor, as it is when the projection runs as a step of its own.
 * x [rows][kdim], w [n_out][kdim] (one row of weights per output channel), v [rows][n_out].
 */
int orc_project(const uint16_t *x, const uint16_t *w, int dtype, int rows, int kdim, int n_out, uint16_t *v)
{
    if (rows < 0 || kdim <= 0 || n_out <= 0) return -1;
    for (int r = 0; r < rows; r++)
        for (int o = 0; o < n_out; o++) {
            double acc = 0.0;
            for (int k = 0; k < kdim; k++)
                acc += (double)widen(x[(size_t)r * kdim + k], dtype) * (double)widen(w[(size_t)o * kdim + k], dtype);
            v[(size_t)r * n_out + o] = orc_f64_to_16_rne(acc, dtype);
        }
    return 0;
}

/* The same dot products before the rounding, and the sums of the products' magnitudes (what a
   test needs to bound the error of an implementation that accumulates in a narrower type). */
int orc_project_f64(const uint16_t *x, const uint16_t *w, int dtype, int rows, int kdim, int n_out,
                    double *sum, double *abs_sum)
{
    if (rows < 0 || kdim <= 0 || n_out <= 0) return -1;
    for (int r = 0; r < rows; r++)
        for (int o = 0; o < n_out; o++) {
            double acc = 0.0, mag = 0.0;
            for (int k = 0; k < kdim; k++) {
                const double pr = (double)widen(x[(size_t)r * kdim + k], dtype) * (double)widen(w[(size_t)o * kdim + k], dtype);
                acc += pr;
                mag += fabs(pr);
            }
            sum[(size_t)r * n_out + o] = acc;
            abs_sum[(size_t)r * n_out + o] = mag;
        }
    return 0;
}

/* ------------------------------------------------------------------ encoder */

/* scale / zero of one group of deviations (asymmetric min/max), and its codes.
   dev[i*stride], i < n.  Writes *s16, *z16 and code[i*cstride]. */
static void quantize_group(const float *dev, size_t stride, int n, int qmax,
                           uint16_t *s16, uint16_t *z16, uint8_t *code, size_t cstride)
{
    float mn = dev[0], mx = dev[0];
    for (int i = 1; i < n; i++) {
        float v = dev[(size_t)i * stride];
        if (v < mn) mn = v;
        if (v > mx) mx = v;
    }
    if (mn == 0.0f) mn = 0.0f; /* -0 -> +0 so the metadata bits do not depend on scan order */
    if (mx == 0.0f) mx = 0.0f;
    uint16_t zb = orc_f32_to_f16_down(mn);
    float z = orc_f16_to_f32(zb);
    float rng = mx - z;
    float s32 = rng / (float)qmax;
    uint16_t sb = orc_f32_to_f16_up(s32);
    float s = orc_f16_to_f32(sb);
    *s16 = sb;
    *z16 = zb;
    for (int i = 0; i < n; i++) {
        int c = 0;
        if (s != 0.0f) {
            float u = (dev[(size_t)i * stride] - z) / s;
            float r = rintf(u); /* round to nearest, ties to even (default rounding mode) */
            if (r < 0.0f) r = 0.0f;
            if (r > (float)qmax) r = (float)qmax;
            c = (int)r;
        }
        code[(size_t)i * cstride] = (uint8_t)c;
    }
}

/*
 * Encode one block of G tokens of one batch element (all H kv heads).
 * bits in {2,4,8}.  Returns 0, or -1 on a bad argument.
 */
int orc_encode_block(const uint16_t *x, int dtype, int G, int H, int d, int Gc, int bits,
                     int mean_mode, int which,
                     uint8_t *codes, uint16_t *scale, uint16_t *zero, uint16_t *mean)
{
    if (!x || !codes || !scale || !zero) return -1;
    if (!(bits == 2 || bits == 4 || bits == 8)) return -1;
    if (G <= 0 || H <= 0 || d <= 0 || Gc <= 0 || d % Gc) return -1;
    if (mean_mode != ORC_MEAN_NONE && !mean) return -1;
    const int qmax = (1 << bits) - 1;
    float *dev = (float *)malloc(sizeof(float) * (size_t)G * H * d); /* [H][G][d] */
    if (!dev) return -1;

    /* Step 1-2: mean (Eq. 1-2; read as the arithmetic mean) and deviation (Eq. 3-4). */
    for (int h = 0; h < H; h++)
        for (int t = 0; t < G; t++)
            for (int c = 0; c < d; c++)
                dev[((size_t)h * G + t) * d + c] = widen(x[((size_t)t * H + h) * d + c], dtype);

    if (mean_mode == ORC_MEAN_CHANNEL_BLOCK) {
        for (int h = 0; h < H; h++)
            for (int c = 0; c < d; c++) {
                float acc = 0.0f;
                for (int t = 0; t < G; t++) acc = acc + dev[((size_t)h * G + t) * d + c];
                float m32 = acc / (float)G;
                uint16_t mb = orc_f32_to_f16_rne(m32);
                mean[(size_t)h * d + c] = mb;
                float m = orc_f16_to_f32(mb);
                for (int t = 0; t < G; t++) {
                    size_t i = ((size_t)h * G + t) * d + c;
                    dev[i] = dev[i] - m;
                }
            }
    } else if (mean_mode == ORC_MEAN_CROSS_HEAD) {
        for (int t = 0; t < G; t++)
            for (int c = 0; c < d; c++) {
                float acc = 0.0f;
                for (int h = 0; h < H; h++) acc = acc + dev[((size_t)h * G + t) * d + c];
                float m32 = acc / (float)H;
                uint16_t mb = orc_f32_to_f16_rne(m32);
                mean[(size_t)t * d + c] = mb;
                float m = orc_f16_to_f32(mb);
                for (int h = 0; h < H; h++) {
                    size_t i = ((size_t)h * G + t) * d + c;
                    dev[i] = dev[i] - m;
                }
            }
    } else if (mean_mode != ORC_MEAN_NONE) {
        free(dev);
        return -1;
    }

    /* Step 3-5: group extrema, 16-bit metadata, codes. */
    if (which == ORC_K) {
        /* keys: one group per (head, channel), running over the block's G tokens */
        for (int h = 0; h < H; h++)
            for (int c = 0; c < d; c++)
                quantize_group(dev + (size_t)h * G * d + c, (size_t)d, G, qmax,
                               &scale[(size_t)h * d + c], &zero[(size_t)h * d + c],
                               codes + (size_t)h * G * d + c, (size_t)d);
    } else if (which == ORC_V) {
        /* values: one group per (head, token, channel group of Gc) */
        const int ng = d / Gc;
        for (int h = 0; h < H; h++)
            for (int t = 0; t < G; t++)
                for (int g = 0; g < ng; g++) {
                    size_t o = ((size_t)h * G + t) * d + (size_t)g * Gc;
                    size_t mo = ((size_t)h * G + t) * ng + g;
                    quantize_group(dev + o, 1, Gc, qmax, &scale[mo], &zero[mo], codes + o, 1);
                }
    } else {
        free(dev);
        return -1;
    }
    free(dev);
    return 0;
}

/*
 * Reconstruction of one block (Eq. 7-8 with the sign convention above):
 * x^ = mean + (zero + scale * code), evaluated in binary32 in that order.
 * xhat [H][G][d].
 */
int orc_decode_block(const uint8_t *codes, const uint16_t *scale, const uint16_t *zero,
                     const uint16_t *mean, int G, int H, int d, int Gc, int mean_mode,
                     int which, float *xhat)
{
    if (!codes || !scale || !zero || !xhat) return -1;
    const int ng = d / Gc;
    for (int h = 0; h < H; h++)
        for (int t = 0; t < G; t++)
            for (int c = 0; c < d; c++) {
                size_t i = ((size_t)h * G + t) * d + c;
                size_t mi = (which == ORC_K) ? ((size_t)h * d + c)
                                             : (((size_t)h * G + t) * ng + c / Gc);
                float s = orc_f16_to_f32(scale[mi]);
                float z = orc_f16_to_f32(zero[mi]);
                float deq = s * (float)codes[i];
                deq = z + deq;
                float m = 0.0f;
                if (mean_mode == ORC_MEAN_CHANNEL_BLOCK) m = orc_f16_to_f32(mean[(size_t)h * d + c]);
                else if (mean_mode == ORC_MEAN_CROSS_HEAD) m = orc_f16_to_f32(mean[(size_t)t * d + c]);
                xhat[i] = m + deq;
            }
    return 0;
}

/* ------------------------------------------------------------------ bit packing */

/*
 * Physical position of the code of (token t, channel c) inside one head's packed block.
 * A block is cut into 16 x 16 tiles of codes ("line" x "slot").  A line's 16 slots sit in
 * 2*bits consecutive bytes, i.e. bits/2 32-bit words of 32/bits slots each.  Inside a word the
 * slots are byte-interleaved: the word's slot number 4*f + y (y = 0..3) is field f of byte y,
 * field f being bits [bits*f, bits*f + bits) of that byte.  Sixteen bytes ("piece") hold the
 * same line of 8/bits tiles; sixteen pieces (lines 0..15) are consecutive.
 * Keys: line = token, slot = channel; a piece holds channel tiles (2j, 2j+1) at 4 bits, those
 * two tiles for two consecutive token tiles at 2 bits, and one tile at 8 bits, where pieces
 * are ordered (token tile, tile parity, j).  Values: line = channel, slot = token.
 * d must be 128 (eight channel tiles).  G is a multiple of 16 (32 for 2-bit keys).
 */
static void slot_in_line(int bits, int e, size_t *byte_in_line, int *shift)
{
    const int per_word = 32 / bits;          /* slots per 32-bit word */
    const int word = e / per_word, r = e % per_word;
    *byte_in_line = (size_t)word * 4 + (size_t)(r % 4);
    *shift = bits * (r / 4);
}

static void code_position(int which, int bits, int G, int t, int c, size_t *byte, int *shift)
{
    size_t piece, tile_off, in_line;
    const int line_bytes = 2 * bits; /* bytes of one tile line */
    if (which == ORC_K) {
        int tt = t / 16, n = t % 16, cg = c / 16, e = c % 16;
        slot_in_line(bits, e, &in_line, shift);
        if (bits == 8) {
            piece = ((size_t)(tt * 2 + cg % 2) * 4 + cg / 2) * 16 + n;
            tile_off = 0;
        } else if (bits == 4) {
            piece = ((size_t)tt * 4 + cg / 2) * 16 + n;
            tile_off = (size_t)(cg % 2) * line_bytes;
        } else {
            piece = ((size_t)(tt / 2) * 4 + cg / 2) * 16 + n;
            tile_off = (size_t)((tt % 2) * 2 + cg % 2) * line_bytes;
        }
    } else {
        int tt = t / 16, e = t % 16, ct = c / 16, n = c % 16, nt = G / 16;
        slot_in_line(bits, e, &in_line, shift);
        if (bits == 8) {
            piece = ((size_t)ct * nt + tt) * 16 + n;
            tile_off = 0;
        } else if (bits == 4) {
            piece = ((size_t)(ct / 2) * nt + tt) * 16 + n;
            tile_off = (size_t)(ct % 2) * line_bytes;
        } else {
            piece = ((size_t)(ct / 4) * nt + tt) * 16 + n;
            tile_off = (size_t)(ct % 4) * line_bytes;
        }
    }
    *byte = piece * 16 + tile_off + in_line;
}

/* codes [G][d] of one head -> packed [G*d*bits/8] bytes */
int orc_pack_codes(const uint8_t *codes, int which, int bits, int G, int d, uint8_t *packed)
{
    if (!codes || !packed || d != 128 || G % 16) return -1;
    if (!(bits == 2 || bits == 4 || bits == 8)) return -1;
    if (which == ORC_K && bits == 2 && G % 32) return -1;
    memset(packed, 0, (size_t)G * d * bits / 8);
    for (int t = 0; t < G; t++)
        for (int c = 0; c < d; c++) {
            size_t byte; int shift;
            code_position(which, bits, G, t, c, &byte, &shift);
            packed[byte] |= (uint8_t)(codes[(size_t)t * d + c] << shift);
        }
    return 0;
}

int orc_unpack_codes(const uint8_t *packed, int which, int bits, int G, int d, uint8_t *codes)
{
    if (!codes || !packed || d != 128 || G % 16) return -1;
    if (!(bits == 2 || bits == 4 || bits == 8)) return -1;
    if (which == ORC_K && bits == 2 && G % 32) return -1;
    for (int t = 0; t < G; t++)
        for (int c = 0; c < d; c++) {
            size_t byte; int shift;
            code_position(which, bits, G, t, c, &byte, &shift);
            codes[(size_t)t * d + c] = (uint8_t)((packed[byte] >> shift) & ((1 << bits) - 1));
        }
    return 0;
}

/* ------------------------------------------------------------------ attention */

/*
 * Softmax attention of g query heads against one kv head (Eq. 5-6), binary64:
 *   a_t = softmax_t( q . k_t / sqrt(d) ),  o = sum_t a_t v_t.
 * k, v are the reconstructed (or raw residual) rows, already in token order
 * (Eq. 9-10: compressed head of the sequence followed by the raw tail).
 * q [g][d], k [T][d], v [T][d], out [g][d].
 */
int orc_attention(const double *q, const float *k, const float *v, int T, int d, int g,
                  double *out)
{
    if (!q || !k || !v || !out || T <= 0 || d <= 0 || g <= 0) return -1;
    double *sc = (double *)malloc(sizeof(double) * (size_t)T);
    if (!sc) return -1;
    const double inv = 1.0 / sqrt((double)d);
    for (int i = 0; i < g; i++) {
        double mx = -INFINITY;
        for (int t = 0; t < T; t++) {
            double acc = 0.0;
            for (int c = 0; c < d; c++) acc += q[(size_t)i * d + c] * (double)k[(size_t)t * d + c];
            sc[t] = acc * inv;
            if (sc[t] > mx) mx = sc[t];
        }
        double den = 0.0;
        for (int t = 0; t < T; t++) { sc[t] = exp(sc[t] - mx); den += sc[t]; }
        for (int c = 0; c < d; c++) {
            double acc = 0.0;
            for (int t = 0; t < T; t++) acc += sc[t] * (double)v[(size_t)t * d + c];
            out[(size_t)i * d + c] = acc / den;
        }
    }
    free(sc);
    return 0;
}

/* widen a run of 16-bit values to binary32 (raw residual tokens, 16-bit passthrough) */
void orc_widen(const uint16_t *x, int dtype, size_t n, float *out)
{
    for (size_t i = 0; i < n; i++) out[i] = widen(x[i], dtype);
}
