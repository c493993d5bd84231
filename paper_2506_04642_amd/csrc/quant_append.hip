// Quantise-and-append kernels (gfx950).
//
// flush_block_kernel compresses one block of G tokens of one (sequence, kv head) for keys or for
// values: mean-centring (arxiv 2506.04642 Sec. 3.1, Eq. 1-2, taken here per channel over the
// block), deviation (Sec. 3.2, Eq. 3-4), asymmetric min/max group quantisation of the deviation
// with binary16 scale / zero (the S and M of Algorithm 1), and bit-packing into the tiled
// storage format.  Keys are grouped per channel over the block's tokens, values per token over
// groups of Gc channels.
//
// The arithmetic is IEEE binary32, one rounding per operation in a fixed order (this file is
// compiled with -ffp-contract=off), so that the bytes written are reproducible bit for bit:
//   mean  = f16_rne( (x_0 + x_1 + ... + x_{G-1}) / G )        sequential sum in token order
//   D     = x - mean
//   zero  = f16_round_down(min D)   scale = f16_round_up((max D - zero) / qmax)
//   code  = clamp(rint((D - zero) / scale), 0, qmax)          0 when scale == 0
//
// resid_copy_kernel stores raw 16-bit tokens in the residual buffer (Sec. 3.3).
//
// With rotary tables (Algorithm 1 step 5: rotation fused with the key compression) every kernel
// turns the new key rows on their way in, in binary32 with one rounding per operation,
//   y_a = x_a cos - x_b sin     y_b = x_b cos + x_a sin
// and rounds the result to the 16-bit type, so that the cache holds exactly what a separate
// rotation step followed by a plain append would have stored.
#include "quant_wave.h"

namespace tadakv {
namespace {

constexpr int kThreads = 256;
constexpr int kRowPad = kHeadDim + 4; // floats per LDS row: rows stay 16-byte aligned and start in different banks

// Row of 128 16-bit elements that holds token `ci` of the concatenation
// [old residual (r_old tokens) | new tokens] for unit (b, h).
__device__ __forceinline__ const uint16_t *src_row(const AppendArgs &a, int which, int b, int h, int ci)
{
    const int u = (a.b0 + b) * a.n_kv_heads + h; // unit in the cache
    if (ci < a.r_old) {
        const long long off = (which == 0 ? a.geom.k_resid_off : a.geom.v_resid_off) +
                              ((long long)u * a.geom.R + ci) * (kHeadDim * 2);
        return (const uint16_t *)(a.layer + off);
    }
    const uint16_t *base = which == 0 ? a.k_new : a.v_new;
    return base + (long long)b * a.stride_b + (long long)(ci - a.r_old) * a.stride_t + (long long)h * a.stride_h;
}

// A decode step's token, one per sequence, into the raw buffers, with the lengths on the device
// (dev_len): unit u's rows go to position "raw tokens" of its sequence's current state, and the
// state after the step goes to the other slot -- the token counted in, or, if it fills the raw
// buffer, the buffer's tokens counted as packed blocks (the quantiser, launched next, compresses
// them, in the same launch: flush_wave_kernel).  A sequence that has no room left keeps its state
// and takes no token.  A group of 32 threads serves a unit.
__device__ __forceinline__ void step_store_unit(const AppendArgs &a, int u)
{
    const int b = u / a.n_kv_heads, h = u % a.n_kv_heads;
    const int lane = threadIdx.x & 31, which = lane >> 4, ch = lane & 15;
    const LayerGeom &gm = a.geom;
    int nb, r;
    dev_len(a.len_dev, a.batch, b, 0, gm.NB, gm.R, nb, r);
    const bool ok = r < gm.R && nb * gm.G + r + 1 <= gm.NB * gm.G;
    const bool full = r + 1 == gm.R;
    if (ok) {
        const uint16_t *base = which == 0 ? a.k_new : a.v_new;
        const uint16_t *src = base + (long long)b * a.stride_b + (long long)h * a.stride_h + ch * 8;
        const long long off = (which == 0 ? gm.k_resid_off : gm.v_resid_off) + ((long long)u * gm.R + r) * (kHeadDim * 2) + ch * 16;
        *(uint4 *)(a.layer + off) = *(const uint4 *)src;
    }
    if (h == 0 && lane == 0) {
        int *after = a.len_dev + ((a.len_dev[4 * a.batch] & 1) ^ 1) * 2 * a.batch + 2 * b;
        after[0] = ok && full ? nb + gm.R / gm.G : nb;
        after[1] = ok ? (full ? 0 : r + 1) : r;
    }
}
// (token, channel) of the first code of packed word w and whether the word runs along
// channels (keys) or tokens (values); a word holds 32/bits codes.
__device__ __forceinline__ void word_origin(int which, int bits, int G, int w, int &t0, int &c0)
{
    const int piece = w >> 2, wi = w & 3;
    const int n = piece & 15;
    if (which == 0) {
        if (bits == 8) {
            const int j = (piece >> 4) & 3, par = (piece >> 6) & 1, tt = piece >> 7;
            t0 = tt * 16 + n;
            c0 = (j * 2 + par) * 16 + wi * 4;
        } else if (bits == 4) {
            const int j = (piece >> 4) & 3, tt = piece >> 6;
            t0 = tt * 16 + n;
            c0 = (j * 2 + (wi >> 1)) * 16 + (wi & 1) * 8;
        } else {
            const int j = (piece >> 4) & 3, tp = piece >> 6;
            t0 = (tp * 2 + (wi >> 1)) * 16 + n;
            c0 = (j * 2 + (wi & 1)) * 16;
        }
    } else {
        const int nt = G >> 4;
        const int q = piece >> 4; // = ctile_group * nt + tt
        const int tt = q % nt, cgp = q / nt;
        if (bits == 8) {
            c0 = cgp * 16 + n;
            t0 = tt * 16 + wi * 4;
        } else if (bits == 4) {
            c0 = (cgp * 2 + (wi >> 1)) * 16 + n;
            t0 = tt * 16 + (wi & 1) * 8;
        } else {
            c0 = (cgp * 4 + wi) * 16 + n;
            t0 = tt * 16;
        }
    }
}

// Persistent workgroups: each walks the items (block to flush, unit, K|V) it = blockIdx.x,
// blockIdx.x + gridDim.x, ... and loads the 16-bit rows of its next item into registers before it
// starts the arithmetic of the current one, so that HBM latency is covered by the quantiser.
// All loops have compile-time trip counts: a thread pulls its 16..64 elements out of LDS in one
// burst, works in registers, and writes back in one burst.
template <int G, int GC, bool ROPE>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu((G == 32 && GC == 32) ? 4 : 1, 8))) void flush_block_kernel(AppendArgs a, int n_items)
{
    constexpr int NLD = G * 16 / kThreads;   // 16-byte pieces per thread and item
    constexpr int HT = G / 2;                // tokens per thread in the per-channel passes
    constexpr int NGV = kHeadDim / GC;       // value groups per token
    constexpr int HW = GC / 2;               // channels per thread in the value-group pass
    constexpr int V_ITEMS = G * NGV * 2;     // value groups x two threads each
    constexpr int V_PER = V_ITEMS / kThreads > 0 ? V_ITEMS / kThreads : 1;
    constexpr int MM_N = V_ITEMS > kThreads ? V_ITEMS : kThreads;
    extern __shared__ float lds[];
    const LayerGeom &gm = a.geom;
    float *x = lds;                                            // [G][kRowPad] values, then deviations
    unsigned char *cb = (unsigned char *)(lds + G * kRowPad);  // codes: keys [G][128], values [128][G]
    float *meanv = (float *)(cb + G * kHeadDim);               // [128] channel means
    float *mm = meanv + kHeadDim;                              // [2][MM_N] partial minima, maxima
    const int tid = threadIdx.x;
    const int U = a.batch * a.n_kv_heads;
    const bool centre = gm.mean_mode == 0; // per-channel block mean

    // Item `it` is (block, unit) number it / 2, keys or values.  A workgroup's items are a whole
    // number of grids apart; with an even grid a plain it & 1 would hand it keys only or values
    // only, and the two cost differently, so the side flips from one round of the grid to the next.
    auto side_of = [&](int it) {
        const int round = (gridDim.x & 1) ? 0 : it / (int)gridDim.x;
        return (it ^ round) & 1;
    };
    constexpr int NRP = ROPE ? G * 64 / kThreads : 1; // (token, pair) rotations per thread and key item
    uint4 pre[NLD];
    float pcs[NRP], psn[NRP]; // the angles of the next key item travel with its rows
    auto fetch = [&](int it) {
        const int which = side_of(it), u = (it >> 1) % U, fb = (it >> 1) / U;
        const int b = u / a.n_kv_heads, h = u % a.n_kv_heads;
#pragma unroll
        for (int k = 0; k < NLD; k++) {
            const int i = tid + k * kThreads, t = i >> 4, ch = i & 15;
            pre[k] = *(const uint4 *)(src_row(a, which, b, h, fb * G + t) + ch * 8);
        }
    };
    // The angles of a key item are loaded when its arithmetic starts, ahead of the prefetch of the
    // next item's rows (loads return in order: issued after it they would wait for HBM), and are
    // dead again after the rotation, so they do not add to the register peak of the quantiser.
    auto fetch_angles = [&](int it) {
        const int which = side_of(it), fb = (it >> 1) / U;
        if (ROPE && which == 0) {
#pragma unroll
            for (int k = 0; k < NRP; k++) {
                const int i = tid + k * kThreads, t = i >> 6, pr = i & 63;
                int tn = fb * G + t - a.r_old; // negative: a row from the residual buffer, not turned
                tn = tn < 0 ? 0 : tn;
                pcs[k] = a.rope_cos[(long long)tn * 64 + pr];
                psn[k] = a.rope_sin[(long long)tn * 64 + pr];
            }
        }
    };
    if ((int)blockIdx.x < n_items) fetch(blockIdx.x);

    for (int it = blockIdx.x; it < n_items; it += gridDim.x) {
        const int which = side_of(it), u = (it >> 1) % U, fb = (it >> 1) / U;
        const int b = u / a.n_kv_heads, h = u % a.n_kv_heads;
        const int bits = which == 0 ? gm.k_bits : gm.v_bits;
        unsigned char *rec = a.layer + record_offset(gm, a.n_kv_heads, a.b0 + b, h, a.first_block + fb);
        unsigned char *codes_out = rec + (which == 0 ? gm.k_codes : gm.v_codes);

        if (bits == 16 && !(ROPE && which == 0)) {
            // stored raw: G rows of 256 bytes
#pragma unroll
            for (int k = 0; k < NLD; k++) {
                const int i = tid + k * kThreads, t = i >> 4, ch = i & 15;
                *(uint4 *)(codes_out + (long long)t * 256 + ch * 16) = pre[k];
            }
            if (it + (int)gridDim.x < n_items) fetch(it + gridDim.x);
            continue;
        }

        // 1. the block, widened to binary32, into LDS; then start loading the next item
        fetch_angles(it);
#pragma unroll
        for (int k = 0; k < NLD; k++) {
            const int i = tid + k * kThreads, t = i >> 4, ch = i & 15;
            const uint32_t wv[4] = {pre[k].x, pre[k].y, pre[k].z, pre[k].w};
            float4 lo, hi;
            lo.x = widen16((uint16_t)(wv[0] & 0xFFFFu), gm.dtype); lo.y = widen16((uint16_t)(wv[0] >> 16), gm.dtype);
            lo.z = widen16((uint16_t)(wv[1] & 0xFFFFu), gm.dtype); lo.w = widen16((uint16_t)(wv[1] >> 16), gm.dtype);
            hi.x = widen16((uint16_t)(wv[2] & 0xFFFFu), gm.dtype); hi.y = widen16((uint16_t)(wv[2] >> 16), gm.dtype);
            hi.z = widen16((uint16_t)(wv[3] & 0xFFFFu), gm.dtype); hi.w = widen16((uint16_t)(wv[3] >> 16), gm.dtype);
            *(float4 *)(x + t * kRowPad + ch * 8) = lo;
            *(float4 *)(x + t * kRowPad + ch * 8 + 4) = hi;
        }
        if (it + (int)gridDim.x < n_items) fetch(it + gridDim.x);
        __syncthreads();

        if (ROPE && which == 0) {
            // 1b. turn the key rows that come from this call's input (rows taken from the residual
            // buffer were turned when they were stored); one thread per (token, pair)
            const int pr = tid & 63;
            const int ia = a.rope == 1 ? pr : 2 * pr, ib = a.rope == 1 ? pr + 64 : 2 * pr + 1;
            auto turn = [&](auto dt) {
#pragma unroll
                for (int k = 0; k < NRP; k++) {
                    const int t = (tid >> 6) + k * (kThreads / 64);
                    float ya, yb;
                    rope_pair_t<decltype(dt)::value>(x[t * kRowPad + ia], x[t * kRowPad + ib], pcs[k], psn[k], ya, yb);
                    if (fb * G + t >= a.r_old) {
                        x[t * kRowPad + ia] = ya;
                        x[t * kRowPad + ib] = yb;
                    }
                }
            };
            if (gm.dtype == 1) turn(std::integral_constant<int, 1>{});
            else turn(std::integral_constant<int, 0>{});
            __syncthreads();
            if (bits == 16) {
                // stored raw: the rotated rows, narrowed again (exact)
                for (int i = tid; i < G * 16; i += kThreads) {
                    const int t = i >> 4, ch = i & 15;
                    uint32_t w[4];
#pragma unroll
                    for (int e = 0; e < 4; e++)
                        w[e] = (uint32_t)narrow16(x[t * kRowPad + ch * 8 + 2 * e], gm.dtype) |
                               ((uint32_t)narrow16(x[t * kRowPad + ch * 8 + 2 * e + 1], gm.dtype) << 16);
                    *(uint4 *)(codes_out + (long long)t * 256 + ch * 16) = uint4{w[0], w[1], w[2], w[3]};
                }
                __syncthreads();
                continue;
            }
        }

        const int qmax = (1 << bits) - 1;
        const float qmaxf = (float)qmax;

        // 2. channel mean over the block's tokens: sequential sum in token order, one thread per channel
        if (tid < kHeadDim) {
            const int c = tid;
            float m = 0.0f;
            if (centre) {
                float v[G];
#pragma unroll
                for (int t = 0; t < G; t++) v[t] = x[t * kRowPad + c];
                float acc = 0.0f;
#pragma unroll
                for (int t = 0; t < G; t++) acc = acc + v[t];
                const float m32 = acc / (float)G;
                const uint16_t m16 = f16_rne(m32);
                m = f16_val(m16);
                *(uint16_t *)(rec + (which == 0 ? gm.k_mean : gm.v_mean) + c * 2) = m16;
            }
            meanv[c] = m;
        }
        __syncthreads();

        // 3. deviation; every thread owns half of a channel's tokens
        {
            const int c = tid & 127, half = tid >> 7;
            const int t_lo = half * HT;
            const float mch = meanv[c];
            // cross-head mode: the mean of (token, channel) over the kv heads, written by
            // xhead_mean_kernel just before this launch
            const uint16_t *xm = gm.mean_mode == 1
                                     ? (const uint16_t *)(a.layer + xmean_offset(gm, a.b0 + b, a.first_block + fb, which))
                                     : nullptr;
            float dv[HT];
#pragma unroll
            for (int i = 0; i < HT; i++) dv[i] = x[(t_lo + i) * kRowPad + c];
            float mn = INFINITY, mx = -INFINITY;
#pragma unroll
            for (int i = 0; i < HT; i++) {
                const float m = xm ? f16_val(xm[(t_lo + i) * kHeadDim + c]) : mch;
                dv[i] = dv[i] - m;
                mn = fminf(mn, dv[i]); // a zero of either sign may win; group_meta makes it +0
                mx = fmaxf(mx, dv[i]);
            }
            if (which == 0) {
                // keys: one group per channel over all tokens of the block (extrema are order-free)
                mm[tid] = mn;
                mm[MM_N + tid] = mx;
                __syncthreads();
                const float o_mn = mm[tid ^ 128], o_mx = mm[MM_N + (tid ^ 128)];
                mn = fminf(mn, o_mn);
                mx = fmaxf(mx, o_mx);
                uint16_t s16, z16;
                float sc, z;
                group_meta(mn, mx, qmax, s16, z16, sc, z);
                if (half == 0) {
                    *(uint16_t *)(rec + gm.k_scale + c * 2) = s16;
                    *(uint16_t *)(rec + gm.k_zero + c * 2) = z16;
                }
                const float r = sc != 0.0f ? 1.0f / sc : 0.0f;
#pragma unroll
                for (int i = 0; i < HT; i++)
                    cb[(t_lo + i) * kHeadDim + c] = (unsigned char)quant_code(dv[i], sc, r, z, qmaxf);
            } else {
#pragma unroll
                for (int i = 0; i < HT; i++) x[(t_lo + i) * kRowPad + c] = dv[i];
                __syncthreads();
            }
        }

        if (which == 1) {
            // values: one group per (token, channel group); two threads per group, half the channels
            // each; codes go to LDS transposed ([channel][token]) because value words run along tokens
            float dv[V_PER][HW];
#pragma unroll
            for (int j = 0; j < V_PER; j++) {
                const int idx = tid + j * kThreads;
                if (idx < V_ITEMS) {
                    const int t = idx % G, rest = idx / G, gam = rest % NGV, half = rest / NGV;
                    const float *row = x + t * kRowPad + gam * GC + half * HW;
                    float mn = INFINITY, mx = -INFINITY;
#pragma unroll
                    for (int i = 0; i < HW; i += 4) {
                        const float4 q4 = *(const float4 *)(row + i);
                        dv[j][i] = q4.x; dv[j][i + 1] = q4.y; dv[j][i + 2] = q4.z; dv[j][i + 3] = q4.w;
                    }
#pragma unroll
                    for (int i = 0; i < HW; i++) {
                        mn = fminf(mn, dv[j][i]);
                        mx = fmaxf(mx, dv[j][i]);
                    }
                    mm[idx] = mn;
                    mm[MM_N + idx] = mx;
                }
            }
            __syncthreads();
#pragma unroll
            for (int j = 0; j < V_PER; j++) {
                const int idx = tid + j * kThreads;
                if (idx < V_ITEMS) {
                    const int t = idx % G, rest = idx / G, gam = rest % NGV, half = rest / NGV;
                    const int other = half ? idx - G * NGV : idx + G * NGV;
                    float mn = mm[idx], mx = mm[MM_N + idx];
                    const float o_mn = mm[other], o_mx = mm[MM_N + other];
                    mn = fminf(mn, o_mn);
                    mx = fmaxf(mx, o_mx);
                    uint16_t s16, z16;
                    float sc, z;
                    group_meta(mn, mx, qmax, s16, z16, sc, z);
                    if (half == 0)
                        *(uint32_t *)(rec + gm.v_meta + (t * NGV + gam) * 4) = (uint32_t)s16 | ((uint32_t)z16 << 16);
                    const float r = sc != 0.0f ? 1.0f / sc : 0.0f;
                    unsigned char *col = cb + (gam * GC + half * HW) * G + t;
#pragma unroll
                    for (int i = 0; i < HW; i++) col[i * G] = (unsigned char)quant_code(dv[j][i], sc, r, z, qmaxf);
                }
            }
        }
        __syncthreads();

        // 4. pack.  A 32-bit word holds 32/bits consecutive codes along channels (keys) or tokens
        // (values), byte-interleaved: code number 4f + y is field f of byte y.  In LDS those codes are
        // consecutive bytes, so a word is built from 32-bit reads: w0 | w1 << bits | w2 << 2 bits | ...
        const int n_words = G * kHeadDim * bits / 32;
        const int reads = 8 / bits; // 32-bit reads of four codes per word
        for (int w = tid; w < n_words; w += kThreads) {
            int t0, c0;
            word_origin(which, bits, G, w, t0, c0);
            const uint32_t *src = (const uint32_t *)(which == 0 ? cb + t0 * kHeadDim + c0 : cb + c0 * G + t0);
            uint32_t word = src[0];
            for (int f = 1; f < reads; f++) word |= src[f] << (bits * f);
            ((uint32_t *)codes_out)[w] = word;
        }
        __syncthreads(); // the next item reuses the LDS buffers
    }
}

// ---------------------------------------------------------------------------------------------
// flush_wave_kernel: the same arithmetic for blocks of 32 tokens with one wavefront per item and
// the block held in registers; no LDS, no workgroup barrier.  Lane l owns tokens 8 tg .. 8 tg + 7
// (tg = l & 3) of channels 8 c8 .. 8 c8 + 7 (c8 = l >> 2): a wave's load instruction covers four
// whole rows; the quad holds a channel's 32 tokens, so the token-order sum of the mean and the key
// groups' extrema move by quad DPP; a value group (one token, Gc channels) is lanes 4 apart in a
// row of 16; an 8-token run of one channel (a value word at 4 bits) and 8 channels of one token
// (a key word at 4 bits) are both in one lane.
template <int GC, int BITS, bool ROPE>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(3, 8))) void flush_wave_kernel(AppendArgs a, int n_items)
{
    constexpr int G = 32;
    constexpr int bits = BITS; // the width of the items this launch handles (both sides of a layer with one width, or one side)
    constexpr int NGV = kHeadDim / GC;
    const LayerGeom &gm = a.geom;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int tg = lane & 3, c8 = lane >> 2;
    const int U = a.batch * a.n_kv_heads;
    const int workers = (int)gridDim.x * (kThreads / 64);
    // Each wave assembles its item's part of the record (codes, scale / zero, mean: contiguous in
    // the record) in LDS at the final offsets and then writes it out as one linear run of 16-byte
    // pieces; the words a lane produces are 4 to 16 bytes apart from its neighbours', and storing
    // them directly left partly written cache lines to be completed from memory.
    // (The same buffer first holds the block's raw rows, 8 KiB, for the token-order sum of the mean.)
    constexpr int IMG_BYTES = G * kHeadDim * BITS / 8 + 768 > G * kHeadDim * 2 ? G * kHeadDim * BITS / 8 + 768 : G * kHeadDim * 2;
    __shared__ __attribute__((aligned(16))) unsigned char lds_img[kThreads / 64][IMG_BYTES];
    unsigned char *img = lds_img[wave];

    // a decode step on device-resident lengths: first the step's token goes into the raw buffers and
    // the lengths after the step are written (nothing below reads what this writes: a buffer that the
    // token fills is compressed from its first rows and the caller's row)
    if (a.len_dev)
        for (int su = (int)blockIdx.x * 8 + (int)(threadIdx.x >> 5); su < U; su += (int)gridDim.x * 8) step_store_unit(a, su);

    for (int it = (int)blockIdx.x * (kThreads / 64) + wave; it < n_items; it += workers) {
        // keys and values cost differently: a worker alternates between them (workers is even)
        // (a call that handles one side only numbers its items (block, unit) and takes that side of each)
        const int which = a.sides ? a.sides - 1 : (it ^ (it / workers)) & 1, iu = a.sides ? it : it >> 1;
        const int u = iu % U, fb = iu / U;
        const int b = u / a.n_kv_heads, h = u % a.n_kv_heads;
        int first_block = a.first_block;
        if (a.len_dev) {
            // a decode step on device-resident lengths: the sequence's raw buffer is compressed only if
            // the step's token has filled it (the state before the step says so), as its next blocks
            int nb, r;
            dev_len(a.len_dev, a.batch, b, 0, gm.NB, gm.R, nb, r);
            if (r + 1 != gm.R || nb * G + r + 1 > gm.NB * G) continue;
            first_block = nb;
        }
        unsigned char *rec = a.layer + record_offset(gm, a.n_kv_heads, a.b0 + b, h, first_block + fb);
        const int base_off = which == 0 ? gm.k_codes : gm.v_codes; // start of this item's part of the record
        unsigned char *codes_out = img;

        uint4 pre[8];
        if (fb * G >= a.r_old) {
            // the whole block comes from the call's input (every block but a call's first): one
            // address, the lane's other rows a token stride apart
            const uint16_t *row0 = src_row(a, which, b, h, fb * G + 8 * tg) + c8 * 8;
#pragma unroll
            for (int j = 0; j < 8; j++) pre[j] = *(const uint4 *)(row0 + (long long)j * a.stride_t);
        } else {
#pragma unroll
            for (int j = 0; j < 8; j++) pre[j] = *(const uint4 *)(src_row(a, which, b, h, fb * G + 8 * tg + j) + c8 * 8);
        }

        // ---- per-channel block mean, the sum: over the tokens in order
        uint32_t mean_pair = 0u; // binary16 means of channels 2 lane and 2 lane + 1
        if (gm.mean_mode == 0 && !ROPE) {
            // The raw rows go through LDS ([token][sixteen 16-byte pieces], the pieces of a row
            // rotated by four per eight tokens so that the four lanes of a quad, whose rows lie
            // 2 KiB apart, write to different banks) and come back with a channel pair's 32 tokens
            // in one lane (lane l: channels 2 l and 2 l + 1; one whole row per read instruction):
            // every lane adds, instead of a quarter of them at a time.  The wave's LDS operations
            // complete in the order issued.
            const int piece_w = (c8 + 4 * tg) & 15;
#pragma unroll
            for (int j = 0; j < 8; j++) *(uint4 *)(img + (8 * tg + j) * 256 + piece_w * 16) = pre[j];
            float s0 = 0.0f, s1 = 0.0f;
            const unsigned char *rd = img + (lane & 3) * 4;
            // (eight rows at a time: all 32 reads at once would hold 32 more registers)
#pragma unroll 1
            for (int tq = 0; tq < G / 8; tq++) {
                const unsigned char *rq = rd + tq * 2048 + ((((lane >> 2) + 4 * tq) & 15) << 4);
                uint32_t w[8];
#pragma unroll
                for (int k = 0; k < 8; k++) w[k] = *(const uint32_t *)(rq + k * 256);
                if (gm.dtype == 1) {
#pragma unroll
                    for (int k = 0; k < 8; k++) {
                        s0 = s0 + __uint_as_float(w[k] << 16);
                        s1 = s1 + __uint_as_float(w[k] & 0xFFFF0000u);
                    }
                } else {
#pragma unroll
                    for (int k = 0; k < 8; k++) {
                        s0 = s0 + f16_val((uint16_t)(w[k] & 0xFFFFu));
                        s1 = s1 + f16_val((uint16_t)(w[k] >> 16));
                    }
                }
            }
            mean_pair = (uint32_t)f16_rne(s0 / (float)G) | ((uint32_t)f16_rne(s1 / (float)G) << 16);
        }

        float x[8][8]; // [token j][channel e]
        widen_pieces(pre, gm.dtype, x);

        if (ROPE && which == 0) {
            const int tn0 = fb * G + 8 * tg - a.r_old; // index of this lane's first token in the call's input
            if (gm.dtype == 1) rope_in_lanes<1>(x, a, tn0, lane);
            else rope_in_lanes<0>(x, a, tn0, lane);
        }

        // ---- mean-centring
        if (gm.mean_mode == 0) {
            // per channel over the block: the sum runs over the tokens in order
            float m[8];
            const int mean_off = (which == 0 ? gm.k_mean : gm.v_mean) - base_off;
            if (ROPE) {
                // (the instance that rotates the keys, which then exist in registers only) the four
                // lanes of a quad add their eight tokens one after the other and hand the running sum on
                float acc[8];
#pragma unroll
                for (int e = 0; e < 8; e++) acc[e] = 0.0f;
#pragma unroll
                for (int p = 0; p < 4; p++) {
                    float cin[8];
#pragma unroll
                    for (int e = 0; e < 8; e++)
                        cin[e] = p == 0 ? 0.0f : (p == 1 ? quad_bcast_f<0>(acc[e]) : (p == 2 ? quad_bcast_f<1>(acc[e]) : quad_bcast_f<2>(acc[e])));
                    if (tg == p) {
#pragma unroll
                        for (int e = 0; e < 8; e++) {
                            float sacc = cin[e];
#pragma unroll
                            for (int j = 0; j < 8; j++) sacc = sacc + x[j][e];
                            acc[e] = sacc;
                        }
                    }
                }
                uint32_t mpk[4];
#pragma unroll
                for (int e = 0; e < 8; e++) {
                    const uint32_t m16 = quad_bcast_u<3>((uint32_t)f16_rne(acc[e] / (float)G));
                    m[e] = f16_val((uint16_t)m16);
                    if (e & 1) mpk[e >> 1] |= m16 << 16;
                    else mpk[e >> 1] = m16;
                }
                if (tg == 0) *(uint4 *)(img + mean_off + c8 * 16) = uint4{mpk[0], mpk[1], mpk[2], mpk[3]};
            } else {
                // (summed above, while only the raw rows were held) the record's mean row is the lanes'
                // words in order
                const uint32_t mp = mean_pair;
                *(uint32_t *)(img + mean_off + lane * 4) = mp;
                // channels 8 c8 + 2 k and + 2 k + 1 are quad lane k's
                const uint32_t q0 = quad_bcast_u<0>(mp), q1 = quad_bcast_u<1>(mp), q2 = quad_bcast_u<2>(mp), q3 = quad_bcast_u<3>(mp);
                m[0] = f16_val((uint16_t)(q0 & 0xFFFFu)); m[1] = f16_val((uint16_t)(q0 >> 16));
                m[2] = f16_val((uint16_t)(q1 & 0xFFFFu)); m[3] = f16_val((uint16_t)(q1 >> 16));
                m[4] = f16_val((uint16_t)(q2 & 0xFFFFu)); m[5] = f16_val((uint16_t)(q2 >> 16));
                m[6] = f16_val((uint16_t)(q3 & 0xFFFFu)); m[7] = f16_val((uint16_t)(q3 >> 16));
            }
#pragma unroll
            for (int j = 0; j < 8; j++)
#pragma unroll
                for (int e = 0; e < 8; e++) x[j][e] = x[j][e] - m[e];
        } else if (gm.mean_mode == 1) {
            // mean over the kv heads per (token, channel), written by xhead_mean_kernel before this launch
            const uint16_t *xm = (const uint16_t *)(a.layer + xmean_offset(gm, a.b0 + b, first_block + fb, which));
#pragma unroll
            for (int j = 0; j < 8; j++) {
                const uint4 mv = *(const uint4 *)(xm + (8 * tg + j) * kHeadDim + c8 * 8);
                const uint32_t wv[4] = {mv.x, mv.y, mv.z, mv.w};
#pragma unroll
                for (int k = 0; k < 4; k++) {
                    x[j][2 * k] = x[j][2 * k] - f16_val((uint16_t)(wv[k] & 0xFFFFu));
                    x[j][2 * k + 1] = x[j][2 * k + 1] - f16_val((uint16_t)(wv[k] >> 16));
                }
            }
        } else {
#pragma unroll
            for (int j = 0; j < 8; j++)
#pragma unroll
                for (int e = 0; e < 8; e++) x[j][e] = x[j][e] - 0.0f;
        }

        constexpr int qmax = (1 << bits) - 1;

        if (which == 0) {
            // ---- keys: one group per channel over the 32 tokens (eight in the lane, four lanes)
            float mn[8], mx[8];
#pragma unroll
            for (int e = 0; e < 8; e++) {
                float lo = vmin(vmin3(x[0][e], x[1][e], x[2][e]), vmin3(x[3][e], x[4][e], vmin3(x[5][e], x[6][e], x[7][e])));
                float hi = vmax(vmax3(x[0][e], x[1][e], x[2][e]), vmax3(x[3][e], x[4][e], vmax3(x[5][e], x[6][e], x[7][e])));
                lo = vmin(lo, dpp_f<0xB1>(lo));
                hi = vmax(hi, dpp_f<0xB1>(hi));
                mn[e] = vmin(lo, dpp_f<0x4E>(lo));
                mx[e] = vmax(hi, dpp_f<0x4E>(hi));
            }
            // quad lane tg works out the metadata of channels 2 tg and 2 tg + 1, then all share
            const MetaOut ma = meta_of(pick4(tg, mn[0], mn[2], mn[4], mn[6]), pick4(tg, mx[0], mx[2], mx[4], mx[6]), qmax);
            const MetaOut mb = meta_of(pick4(tg, mn[1], mn[3], mn[5], mn[7]), pick4(tg, mx[1], mx[3], mx[5], mx[7]), qmax);
            uint32_t pk[8];
            float rs[8];
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
                *(uint4 *)(img + (gm.k_scale - base_off) + c8 * 16) = uint4{sw[0], sw[1], sw[2], sw[3]};
                *(uint4 *)(img + (gm.k_zero - base_off) + c8 * 16) = uint4{zw[0], zw[1], zw[2], zw[3]};
            }
            float sc[8], z[8];
#pragma unroll
            for (int e = 0; e < 8; e++) {
                sc[e] = f16_val((uint16_t)(pk[e] & 0xFFFFu));
                z[e] = f16_val((uint16_t)(pk[e] >> 16));
            }
            // codes and words: a key word runs along channels
            const int tt = tg >> 1, jj = c8 >> 2;
#pragma unroll
            for (int j = 0; j < 8; j++) {
                const int n = 8 * (tg & 1) + j;
                float uq[8];
#pragma unroll
                for (int e = 0; e < 8; e++) uq[e] = quant_quotient(x[j][e], sc[e], rs[e], z[e]);
                const uint32_t clo = pack4_u8(uq[0], uq[1], uq[2], uq[3]), chi = pack4_u8(uq[4], uq[5], uq[6], uq[7]);
                if (bits == 8) {
                    const int piece = ((tt * 2 + ((c8 >> 1) & 1)) * 4 + jj) * 16 + n;
                    *(uint2 *)(codes_out + (piece * 4 + 2 * (c8 & 1)) * 4) = uint2{clo, chi};
                } else if (bits == 4) {
                    const uint32_t w = clo | (chi << 4); // byte y: codes y and y + 4
                    ((uint32_t *)codes_out)[((tt * 4 + jj) * 16 + n) * 4 + (c8 & 3)] = w;
                } else {
                    // 16 channels per word: this lane's half, shifted into place, joined with the
                    // neighbouring channel octet's (lane ^ 4)
                    uint32_t w = clo | (chi << 2); // byte y: codes y and y + 4 in its low four bits
                    w <<= 4 * (c8 & 1);
                    w |= from_lane_u(w, lane ^ 4);
                    if ((j >> 2) == (c8 & 1))
                        ((uint32_t *)codes_out)[(jj * 16 + n) * 4 + ((tt << 1) | ((c8 >> 1) & 1))] = w;
                }
            }
        } else {
            // ---- values: one group per (token, Gc channels): eight in the lane, Gc / 8 lanes
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
                const int gam = c8 / (GC / 8), t = 8 * tg + 2 * q4;
                *(uint32_t *)(img + (gm.v_meta - base_off) + (t * NGV + gam) * 4) = ma.pk;
                *(uint32_t *)(img + (gm.v_meta - base_off) + ((t + 1) * NGV + gam) * 4) = mb.pk;
            }
            uint32_t pk[8];
            float rs[8];
#pragma unroll
            for (int j = 0; j < 8; j++) {
                const int src = (lane & ~12) | ((j >> 1) << 2);
                pk[j] = from_lane_u((j & 1) ? mb.pk : ma.pk, src);
                rs[j] = from_lane_f((j & 1) ? mb.rs : ma.rs, src);
            }
            float sc[8], z[8];
#pragma unroll
            for (int j = 0; j < 8; j++) {
                sc[j] = f16_val((uint16_t)(pk[j] & 0xFFFFu));
                z[j] = f16_val((uint16_t)(pk[j] >> 16));
            }
            // codes and words: a value word runs along tokens
            const int tt = tg >> 1;
#pragma unroll
            for (int e = 0; e < 8; e++) {
                const int n = 8 * (c8 & 1) + e;
                float uq[8];
#pragma unroll
                for (int j = 0; j < 8; j++) uq[j] = quant_quotient(x[j][e], sc[j], rs[j], z[j]);
                const uint32_t clo = pack4_u8(uq[0], uq[1], uq[2], uq[3]), chi = pack4_u8(uq[4], uq[5], uq[6], uq[7]);
                if (bits == 8) {
                    const int piece = ((c8 >> 1) * 2 + tt) * 16 + n;
                    *(uint2 *)(codes_out + (piece * 4 + 2 * (tg & 1)) * 4) = uint2{clo, chi};
                } else if (bits == 4) {
                    const uint32_t w = clo | (chi << 4); // byte y: codes y and y + 4
                    const int piece = ((c8 >> 2) * 2 + tt) * 16 + n;
                    ((uint32_t *)codes_out)[piece * 4 + 2 * ((c8 >> 1) & 1) + (tg & 1)] = w;
                } else {
                    uint32_t w = clo | (chi << 2); // byte y: codes y and y + 4 in its low four bits
                    w <<= 4 * (tg & 1);
                    w |= dpp_u<0xB1>(w);
                    const int piece = ((c8 >> 3) * 2 + tt) * 16 + n;
                    if ((e >> 2) == (tg & 1)) ((uint32_t *)codes_out)[piece * 4 + ((c8 >> 1) & 3)] = w;
                }
            }
        }

        // ---- the assembled part of the record -> memory, linear
        int part_bytes;
        if (which == 0) part_bytes = (gm.mean_mode == 0 ? gm.k_mean : gm.k_zero) + 256 - base_off;
        else part_bytes = (gm.mean_mode == 0 ? gm.v_mean + 256 : gm.v_meta + G * NGV * 4) - base_off;
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); // this wave's LDS writes have landed
        for (int off = lane * 16; off < part_bytes; off += 64 * 16) *(uint4 *)(rec + base_off + off) = *(const uint4 *)(img + off);
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); // the image is in registers before the next item overwrites it
    }
}


// The same for blocks of 64 or 128 tokens: a wave takes the block in parts of 32 tokens, twice.
// The first pass gathers what spans the block -- the per-channel sums in token order (the
// running sum goes from quad lane 3 of one part to quad lane 0 of the next) and, for
// keys, the channels' extrema --, the second pass loads the rows again (they are in the cache),
// forms the deviations and emits metadata, codes and words part by part.  With a per-channel
// mean m the extrema of the deviations are those of the raw values moved by m: rounding is
// monotone, so min_t fl(x_t - m) = fl(min_t x_t - m).
template <int G, int GC, int BITS, bool ROPE> struct WaveImage {
    static constexpr int NGV = kHeadDim / GC;
    static constexpr int META_BYTES = G * NGV * 4 + 256 > 768 ? G * NGV * 4 + 256 : 768;
    static constexpr int BYTES = G * kHeadDim * BITS / 8 + META_BYTES; // the larger of a record's key and value part
};
template <int G, int GC, int BITS, bool ROPE>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(ROPE ? 2 : 3, 8))) void flush_wave_parts_kernel(AppendArgs a, int n_items)
{
    constexpr int NP = G / 32; // parts of 32 tokens
    constexpr int NGV = kHeadDim / GC;
    constexpr int qmax = (1 << BITS) - 1;
    const LayerGeom &gm = a.geom;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int tg = lane & 3, c8 = lane >> 2;
    const int U = a.batch * a.n_kv_heads;
    const int workers = (int)gridDim.x * (kThreads / 64);
    constexpr int IMG_BYTES = WaveImage<G, GC, BITS, ROPE>::BYTES;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_img[]; // [waves][IMG_BYTES], sized at launch
    unsigned char *img = lds_img + wave * IMG_BYTES;

    // a decode step on device-resident lengths (as in flush_wave_kernel): the step's token and the
    // lengths after the step first, then only the raw buffers that the token has filled
    if (a.len_dev)
        for (int su = (int)blockIdx.x * 8 + (int)(threadIdx.x >> 5); su < U; su += (int)gridDim.x * 8) step_store_unit(a, su);

    for (int it = (int)blockIdx.x * (kThreads / 64) + wave; it < n_items; it += workers) {
        const int which = (it ^ (it / workers)) & 1, u = (it >> 1) % U, fb = (it >> 1) / U;
        const int b = u / a.n_kv_heads, h = u % a.n_kv_heads;
        int first_block = a.first_block;
        if (a.len_dev) {
            int nb, r;
            dev_len(a.len_dev, a.batch, b, 0, gm.NB, gm.R, nb, r);
            if (r + 1 != gm.R || nb * G + r + 1 > gm.NB * G) continue;
            first_block = nb;
        }
        unsigned char *rec = a.layer + record_offset(gm, a.n_kv_heads, a.b0 + b, h, first_block + fb);
        const int base_off = which == 0 ? gm.k_codes : gm.v_codes;
        const int mode = gm.mean_mode;
        const uint16_t *xm = mode == 1 ? (const uint16_t *)(a.layer + xmean_offset(gm, a.b0 + b, first_block + fb, which)) : nullptr;

        // rows 32 half + 8 tg .. + 7 of the block, channels 8 c8 .. + 7, widened; in cross-head
        // mode already as deviations from the (token, channel) mean
        auto load_half = [&](int half, float (&x)[8][8]) {
            uint4 pre[8];
#pragma unroll
            for (int j = 0; j < 8; j++) pre[j] = *(const uint4 *)(src_row(a, which, b, h, fb * G + 32 * half + 8 * tg + j) + c8 * 8);
            widen_pieces(pre, gm.dtype, x);
            if (ROPE && which == 0) {
                // both passes turn the rows the same way, so they see the same values
                const int tn0 = fb * G + 32 * half + 8 * tg - a.r_old; // this lane's first token in the call's input
                if (gm.dtype == 1) rope_in_lanes<1>(x, a, tn0, lane);
                else rope_in_lanes<0>(x, a, tn0, lane);
            }
            if (mode == 1) {
#pragma unroll
                for (int j = 0; j < 8; j++) {
                    const uint4 mv = *(const uint4 *)(xm + (32 * half + 8 * tg + j) * kHeadDim + c8 * 8);
                    const uint32_t wv[4] = {mv.x, mv.y, mv.z, mv.w};
#pragma unroll
                    for (int k = 0; k < 4; k++) {
                        x[j][2 * k] = x[j][2 * k] - f16_val((uint16_t)(wv[k] & 0xFFFFu));
                        x[j][2 * k + 1] = x[j][2 * k + 1] - f16_val((uint16_t)(wv[k] >> 16));
                    }
                }
            }
        };

        // ---- first pass: channel sums in token order (per-channel mean mode), key extrema
        float acc[8], mn[8], mx[8];
#pragma unroll
        for (int e = 0; e < 8; e++) {
            acc[e] = 0.0f;
            mn[e] = INFINITY;
            mx[e] = -INFINITY;
        }
        if (mode == 0 || which == 0) {
#pragma unroll
            for (int half = 0; half < NP; half++) {
                float x[8][8];
                load_half(half, x);
                if (mode == 0) {
#pragma unroll
                    for (int p = 0; p < 4; p++) {
                        float cin[8];
#pragma unroll
                        for (int e = 0; e < 8; e++)
                            cin[e] = p == 0 ? (half == 0 ? 0.0f : quad_bcast_f<3>(acc[e]))
                                            : (p == 1 ? quad_bcast_f<0>(acc[e]) : (p == 2 ? quad_bcast_f<1>(acc[e]) : quad_bcast_f<2>(acc[e])));
                        if (tg == p) {
#pragma unroll
                            for (int e = 0; e < 8; e++) {
                                float sacc = cin[e];
#pragma unroll
                                for (int j = 0; j < 8; j++) sacc = sacc + x[j][e];
                                acc[e] = sacc;
                            }
                        }
                    }
                }
                if (which == 0) {
#pragma unroll
                    for (int e = 0; e < 8; e++) {
                        mn[e] = vmin3(vmin3(mn[e], x[0][e], x[1][e]), vmin3(x[2][e], x[3][e], x[4][e]), vmin3(x[5][e], x[6][e], x[7][e]));
                        mx[e] = vmax3(vmax3(mx[e], x[0][e], x[1][e]), vmax3(x[2][e], x[3][e], x[4][e]), vmax3(x[5][e], x[6][e], x[7][e]));
                    }
                }
            }
        }
        float m[8];
#pragma unroll
        for (int e = 0; e < 8; e++) m[e] = 0.0f;
        if (mode == 0) {
            uint32_t mpk[4];
#pragma unroll
            for (int e = 0; e < 8; e++) {
                const uint32_t m16 = quad_bcast_u<3>((uint32_t)f16_rne(acc[e] / (float)G));
                m[e] = f16_val((uint16_t)m16);
                if (e & 1) mpk[e >> 1] |= m16 << 16;
                else mpk[e >> 1] = m16;
            }
            if (tg == 0)
                *(uint4 *)(img + ((which == 0 ? gm.k_mean : gm.v_mean) - base_off) + c8 * 16) = uint4{mpk[0], mpk[1], mpk[2], mpk[3]};
        }

        if (which == 0) {
            // ---- keys: extrema over the quad, moved by the mean; metadata; then the codes
#pragma unroll
            for (int e = 0; e < 8; e++) {
                float lo = mn[e], hi = mx[e];
                lo = vmin(lo, dpp_f<0xB1>(lo));
                hi = vmax(hi, dpp_f<0xB1>(hi));
                lo = vmin(lo, dpp_f<0x4E>(lo));
                hi = vmax(hi, dpp_f<0x4E>(hi));
                mn[e] = lo - m[e];
                mx[e] = hi - m[e];
            }
            float sc[8], rs[8], z[8];
            key_metadata(mn, mx, qmax, lane, img + (gm.k_scale - base_off), img + (gm.k_zero - base_off), sc, rs, z);
#pragma unroll
            for (int half = 0; half < NP; half++) {
                float x[8][8];
                load_half(half, x);
#pragma unroll
                for (int j = 0; j < 8; j++)
#pragma unroll
                    for (int e = 0; e < 8; e++) x[j][e] = x[j][e] - m[e];
                emit_key_words<BITS>(x, sc, rs, z, half, lane, img);
            }
        } else {
#pragma unroll
            for (int half = 0; half < NP; half++) {
                float x[8][8];
                load_half(half, x);
#pragma unroll
                for (int j = 0; j < 8; j++)
#pragma unroll
                    for (int e = 0; e < 8; e++) x[j][e] = x[j][e] - m[e];
                emit_value_half<GC, BITS, G / 16>(x, half, lane, img, img + (gm.v_meta - base_off));
            }
        }

        int part_bytes;
        if (which == 0) part_bytes = (mode == 0 ? gm.k_mean : gm.k_zero) + 256 - base_off;
        else part_bytes = (mode == 0 ? gm.v_mean + 256 : gm.v_meta + G * NGV * 4) - base_off;
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); // this wave's LDS writes have landed
        for (int off = lane * 16; off < part_bytes; off += 64 * 16) *(uint4 *)(rec + base_off + off) = *(const uint4 *)(img + off);
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); // the image is in registers before the next item overwrites it
    }
}

// Blocks of 64 or 128 tokens, one read of the input: the G / 32 wavefronts of a workgroup share an
// item, each with one part of 32 tokens in registers (the lane layout of flush_wave_kernel), and
// exchange through LDS what spans the block.  The per-channel sum of the mean runs over the tokens in
// order, so it passes from part to part: every wave first brings its rows into the layout of the sum
// (through LDS: lane l holds the 32 tokens of channels 2 l and 2 l + 1), then the waves add one after
// the other, each starting from the sum the wave before left in LDS (a barrier per part; the
// workgroups that share the compute unit fill the gaps).  The keys' extrema are those of the parts'.
// Codes, metadata and mean go into one image of the record's key or value part in LDS (it takes the
// place of the raw rows, which nobody needs once the sums are formed), which the waves then write out
// together as one linear run.  For the plain bulk append (no rotation, no device-resident lengths);
// the other calls use flush_wave_parts_kernel, which reads the block twice.
template <int G, int GC, int BITS, bool ROPE>
__global__ __launch_bounds__(64 * (G / 32)) __attribute__((amdgpu_waves_per_eu(ROPE ? 2 : 3, 8))) void flush_coop_kernel(AppendArgs a, int n_items)
{
    constexpr int NP = G / 32; // parts of 32 tokens = waves of the workgroup
    constexpr int NGV = kHeadDim / GC;
    constexpr int qmax = (1 << BITS) - 1;
    constexpr int IMG_BYTES = WaveImage<G, GC, BITS, false>::BYTES;
    constexpr int UNI_BYTES = IMG_BYTES > NP * 8192 ? IMG_BYTES : NP * 8192;
    __shared__ __attribute__((aligned(16))) unsigned char lds_uni[UNI_BYTES]; // raw rows [part][8 KiB], then the image
    __shared__ __attribute__((aligned(16))) float lds_sum[kHeadDim];         // running sums, by channel
    __shared__ __attribute__((aligned(16))) uint32_t lds_mean[kHeadDim / 2]; // the means as binary16 pairs
    __shared__ __attribute__((aligned(16))) float lds_ext[NP][2][kHeadDim];  // the parts' minima and maxima (keys)
    const LayerGeom &gm = a.geom;
    const int lane = threadIdx.x & 63;
    const int part = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int tg = lane & 3, c8 = lane >> 2;
    const int U = a.batch * a.n_kv_heads;
    const int mode = gm.mean_mode;
    unsigned char *img = lds_uni;
    unsigned char *raw = lds_uni + part * 8192;

    // (the grid is even: a workgroup alternates between keys and values, which cost differently, and
    // items 2 j and 2 j + 1 are the two sides of one block)
    for (int it = (int)blockIdx.x; it < n_items; it += (int)gridDim.x) {
        const int which = (it ^ (it / (int)gridDim.x)) & 1, u = (it >> 1) % U, fb = (it >> 1) / U;
        const int b = u / a.n_kv_heads, h = u % a.n_kv_heads;
        unsigned char *rec = a.layer + record_offset(gm, a.n_kv_heads, a.b0 + b, h, a.first_block + fb);
        const int base_off = which == 0 ? gm.k_codes : gm.v_codes;

        // ---- this wave's rows: 32 part + 8 tg .. + 7 of the block, channels 8 c8 .. + 7
        uint4 pre[8];
#pragma unroll
        for (int j = 0; j < 8; j++) pre[j] = *(const uint4 *)(src_row(a, which, b, h, fb * G + 32 * part + 8 * tg + j) + c8 * 8);

        if (ROPE && which == 0) {
            // the key rows of the call are turned here, once (rows from the raw buffer were turned when
            // they were stored), and go back into their 16-bit form, which holds them exactly: what
            // follows takes them as it takes rows that need no turning, and no register keeps the
            // widened values through the sums
            float xr[8][8];
            widen_pieces(pre, gm.dtype, xr);
            const int tn0 = fb * G + 32 * part + 8 * tg - a.r_old; // this lane's first token in the call's input
            if (gm.dtype == 1) rope_in_lanes<1>(xr, a, tn0, lane);
            else rope_in_lanes<0>(xr, a, tn0, lane);
#pragma unroll
            for (int j = 0; j < 8; j++) {
                uint32_t w[4];
#pragma unroll
                for (int q = 0; q < 4; q++)
                    w[q] = gm.dtype == 1 ? pack16_exact<1>(xr[j][2 * q], xr[j][2 * q + 1]) : pack16_exact<0>(xr[j][2 * q], xr[j][2 * q + 1]);
                pre[j] = uint4{w[0], w[1], w[2], w[3]};
            }
        }

        float m[8];
#pragma unroll
        for (int e = 0; e < 8; e++) m[e] = 0.0f;
        if (mode == 0) {
            // the rows in the layout of the sum ([token][sixteen 16-byte pieces], the pieces of a row
            // rotated by four per eight tokens: see flush_wave_kernel), widened
            const int piece_w = (c8 + 4 * tg) & 15;
#pragma unroll
            for (int j = 0; j < 8; j++) *(uint4 *)(raw + (8 * tg + j) * 256 + piece_w * 16) = pre[j];
            float xs0[32], xs1[32];
            const unsigned char *rd = raw + (lane & 3) * 4;
#pragma unroll
            for (int tq = 0; tq < 4; tq++) {
                const unsigned char *rq = rd + tq * 2048 + ((((lane >> 2) + 4 * tq) & 15) << 4);
#pragma unroll
                for (int k = 0; k < 8; k++) {
                    const uint32_t w = *(const uint32_t *)(rq + k * 256);
                    if (gm.dtype == 1) {
                        xs0[8 * tq + k] = __uint_as_float(w << 16);
                        xs1[8 * tq + k] = __uint_as_float(w & 0xFFFF0000u);
                    } else {
                        xs0[8 * tq + k] = f16_val((uint16_t)(w & 0xFFFFu));
                        xs1[8 * tq + k] = f16_val((uint16_t)(w >> 16));
                    }
                }
            }
            // the waves add in turn
#pragma unroll
            for (int p = 0; p < NP; p++) {
                if (part == p) {
                    float s0 = 0.0f, s1 = 0.0f;
                    if (p > 0) {
                        const float2 v = *(const float2 *)&lds_sum[2 * lane];
                        s0 = v.x;
                        s1 = v.y;
                    }
#pragma unroll
                    for (int t = 0; t < 32; t++) {
                        s0 = s0 + xs0[t];
                        s1 = s1 + xs1[t];
                    }
                    if (p < NP - 1) {
                        *(float2 *)&lds_sum[2 * lane] = float2{s0, s1};
                    } else {
                        // (every wave is past its reads of the raw rows: the image may take their place)
                        const uint32_t mp = (uint32_t)f16_rne(s0 / (float)G) | ((uint32_t)f16_rne(s1 / (float)G) << 16);
                        lds_mean[lane] = mp;
                        *(uint32_t *)(img + ((which == 0 ? gm.k_mean : gm.v_mean) - base_off) + lane * 4) = mp;
                    }
                }
                __syncthreads();
            }
            const uint4 mv = *(const uint4 *)&lds_mean[c8 * 4];
            const uint32_t mw[4] = {mv.x, mv.y, mv.z, mv.w};
#pragma unroll
            for (int k = 0; k < 4; k++) {
                m[2 * k] = f16_val((uint16_t)(mw[k] & 0xFFFFu));
                m[2 * k + 1] = f16_val((uint16_t)(mw[k] >> 16));
            }
        }

        // ---- deviations
        float x[8][8]; // [token j][channel e]
        widen_pieces(pre, gm.dtype, x);
        if (mode == 1) {
            // mean over the kv heads per (token, channel), written by xhead_mean_kernel before this launch
            const uint16_t *xm = (const uint16_t *)(a.layer + xmean_offset(gm, a.b0 + b, a.first_block + fb, which));
#pragma unroll
            for (int j = 0; j < 8; j++) {
                const uint4 mv = *(const uint4 *)(xm + (32 * part + 8 * tg + j) * kHeadDim + c8 * 8);
                const uint32_t wv[4] = {mv.x, mv.y, mv.z, mv.w};
#pragma unroll
                for (int k = 0; k < 4; k++) {
                    x[j][2 * k] = x[j][2 * k] - f16_val((uint16_t)(wv[k] & 0xFFFFu));
                    x[j][2 * k + 1] = x[j][2 * k + 1] - f16_val((uint16_t)(wv[k] >> 16));
                }
            }
        }
#pragma unroll
        for (int j = 0; j < 8; j++)
#pragma unroll
            for (int e = 0; e < 8; e++) x[j][e] = x[j][e] - m[e];

        if (which == 0) {
            // ---- keys: one group per channel over the block's tokens: this part's extrema (eight
            // tokens in the lane, four lanes), then all parts'
            float mn[8], mx[8];
#pragma unroll
            for (int e = 0; e < 8; e++) {
                float lo = vmin(vmin3(x[0][e], x[1][e], x[2][e]), vmin3(x[3][e], x[4][e], vmin3(x[5][e], x[6][e], x[7][e])));
                float hi = vmax(vmax3(x[0][e], x[1][e], x[2][e]), vmax3(x[3][e], x[4][e], vmax3(x[5][e], x[6][e], x[7][e])));
                lo = vmin(lo, dpp_f<0xB1>(lo));
                hi = vmax(hi, dpp_f<0xB1>(hi));
                mn[e] = vmin(lo, dpp_f<0x4E>(lo));
                mx[e] = vmax(hi, dpp_f<0x4E>(hi));
            }
            if (tg == 0) {
                *(float4 *)&lds_ext[part][0][8 * c8] = float4{mn[0], mn[1], mn[2], mn[3]};
                *(float4 *)&lds_ext[part][0][8 * c8 + 4] = float4{mn[4], mn[5], mn[6], mn[7]};
                *(float4 *)&lds_ext[part][1][8 * c8] = float4{mx[0], mx[1], mx[2], mx[3]};
                *(float4 *)&lds_ext[part][1][8 * c8 + 4] = float4{mx[4], mx[5], mx[6], mx[7]};
            }
            __syncthreads();
#pragma unroll
            for (int q = 0; q < NP; q++) {
                const float4 l0 = *(const float4 *)&lds_ext[q][0][8 * c8], l1 = *(const float4 *)&lds_ext[q][0][8 * c8 + 4];
                const float4 h0 = *(const float4 *)&lds_ext[q][1][8 * c8], h1 = *(const float4 *)&lds_ext[q][1][8 * c8 + 4];
                const float lv[8] = {l0.x, l0.y, l0.z, l0.w, l1.x, l1.y, l1.z, l1.w};
                const float hv[8] = {h0.x, h0.y, h0.z, h0.w, h1.x, h1.y, h1.z, h1.w};
#pragma unroll
                for (int e = 0; e < 8; e++) {
                    mn[e] = q == 0 ? lv[e] : vmin(mn[e], lv[e]);
                    mx[e] = q == 0 ? hv[e] : vmax(mx[e], hv[e]);
                }
            }
            // (every wave works out the same metadata and stores the same scale / zero rows)
            float sc[8], rs[8], z[8];
            key_metadata(mn, mx, qmax, lane, img + (gm.k_scale - base_off), img + (gm.k_zero - base_off), sc, rs, z);
            emit_key_words<BITS>(x, sc, rs, z, part, lane, img);
        } else {
            emit_value_half<GC, BITS, G / 16>(x, part, lane, img, img + (gm.v_meta - base_off));
        }
        __syncthreads(); // the image is complete

        int part_bytes;
        if (which == 0) part_bytes = (mode == 0 ? gm.k_mean : gm.k_zero) + 256 - base_off;
        else part_bytes = (mode == 0 ? gm.v_mean + 256 : gm.v_meta + G * NGV * 4) - base_off;
        for (int off = (int)threadIdx.x * 16; off < part_bytes; off += NP * 64 * 16)
            *(uint4 *)(rec + base_off + off) = *(const uint4 *)(img + off);
        __syncthreads(); // the image is in registers before the next item's rows overwrite it
    }
}

// Cross-head mean (Eq. 1-2): for every token of a block and every channel, the mean over the kv
// heads, m = f16_rne((x_0 + x_1 + ... + x_{H-1}) / H) with the sum taken in head order.
// grid (blocks to flush, batch, K|V); written to the layer's mean plane.
__global__ __launch_bounds__(kThreads) void xhead_mean_kernel(AppendArgs a)
{
    const LayerGeom &gm = a.geom;
    const int G = gm.G, H = a.n_kv_heads;
    const int fb = blockIdx.x, b = blockIdx.y, which = blockIdx.z;
    const int bits = which == 0 ? gm.k_bits : gm.v_bits;
    if (bits == 16) return;
    int first_block = a.first_block;
    if (a.len_dev) {
        // a decode step on device-resident lengths: only a sequence whose raw buffer the step's token
        // fills gets the rows of its next block(s), as flush_wave_kernel, launched next, compresses only those
        int nb, r;
        dev_len(a.len_dev, a.batch, b, 0, gm.NB, gm.R, nb, r);
        if (r + 1 != gm.R || nb * G + r + 1 > gm.NB * G) return;
        first_block = nb;
    }
    uint16_t *dst = (uint16_t *)(a.layer + xmean_offset(gm, a.b0 + b, first_block + fb, which));
    if (!(a.rope != 0 && which == 0)) {
        // no rotation on this side: a thread takes eight channels of a token as 16-byte pieces
        for (int i = threadIdx.x; i < G * (kHeadDim / 8); i += kThreads) {
            const int t = i / (kHeadDim / 8), c8 = i % (kHeadDim / 8);
            float acc[8];
#pragma unroll
            for (int e = 0; e < 8; e++) acc[e] = 0.0f;
#pragma unroll 4
            for (int h = 0; h < H; h++) {
                const uint4 w = *(const uint4 *)(src_row(a, which, b, h, fb * G + t) + c8 * 8);
                const uint32_t wv[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
                for (int k = 0; k < 4; k++) {
                    acc[2 * k] = acc[2 * k] + widen16((uint16_t)(wv[k] & 0xFFFFu), gm.dtype);
                    acc[2 * k + 1] = acc[2 * k + 1] + widen16((uint16_t)(wv[k] >> 16), gm.dtype);
                }
            }
            uint32_t mw[4];
#pragma unroll
            for (int k = 0; k < 4; k++)
                mw[k] = (uint32_t)f16_rne(acc[2 * k] / (float)H) | ((uint32_t)f16_rne(acc[2 * k + 1] / (float)H) << 16);
            *(uint4 *)(dst + t * kHeadDim + c8 * 8) = uint4{mw[0], mw[1], mw[2], mw[3]};
        }
        return;
    }
    for (int i = threadIdx.x; i < G * (kHeadDim / 2); i += kThreads) {
        const int t = i / (kHeadDim / 2), cp = i % (kHeadDim / 2);
        float acc0 = 0.0f, acc1 = 0.0f;
        const int tn = fb * G + t - a.r_old;
        const bool turn = a.rope != 0 && which == 0 && tn >= 0;
        for (int h = 0; h < H; h++) {
            const uint16_t *row = src_row(a, which, b, h, fb * G + t);
            if (turn) {
                const float *cs = a.rope_cos + (long long)tn * 64, *sn = a.rope_sin + (long long)tn * 64;
                acc0 = acc0 + rope_elem(row, 2 * cp, cs, sn, a.rope, gm.dtype);
                acc1 = acc1 + rope_elem(row, 2 * cp + 1, cs, sn, a.rope, gm.dtype);
            } else {
                const uint32_t w = *(const uint32_t *)(row + 2 * cp);
                acc0 = acc0 + widen16((uint16_t)(w & 0xFFFFu), gm.dtype);
                acc1 = acc1 + widen16((uint16_t)(w >> 16), gm.dtype);
            }
        }
        const uint32_t m0 = f16_rne(acc0 / (float)H), m1 = f16_rne(acc1 / (float)H);
        *(uint32_t *)(dst + t * kHeadDim + 2 * cp) = m0 | (m1 << 16);
    }
}

// Raw tail: input tokens [copy_src, copy_src + copy_n) -> residual rows [copy_dst, ...).
__global__ __launch_bounds__(kThreads) void resid_copy_kernel(AppendArgs a)
{
    const int u = blockIdx.y;
    const int b = u / a.n_kv_heads, h = u % a.n_kv_heads;
    const int i = blockIdx.x * 8 + (threadIdx.x >> 5);
    if (i >= a.copy_n) return;
    const int lane = threadIdx.x & 31, which = lane >> 4, ch = lane & 15;
    if (a.sides && which != a.sides - 1) return;
    const uint16_t *base = which == 0 ? a.k_new : a.v_new;
    const uint16_t *src = base + (long long)b * a.stride_b + (long long)(a.copy_src + i) * a.stride_t +
                          (long long)h * a.stride_h + ch * 8;
    const long long off = (which == 0 ? a.geom.k_resid_off : a.geom.v_resid_off) +
                          ((long long)(a.b0 * a.n_kv_heads + u) * a.geom.R + a.copy_dst + i) * (kHeadDim * 2) + ch * 16;
    if (a.rope != 0 && which == 0) {
        const uint16_t *row = src - ch * 8;
        const int tn = a.copy_src + i;
        const float *cs = a.rope_cos + (long long)tn * 64, *sn = a.rope_sin + (long long)tn * 64;
        uint32_t w[4];
#pragma unroll
        for (int e = 0; e < 4; e++)
            w[e] = (uint32_t)narrow16(rope_elem(row, ch * 8 + 2 * e, cs, sn, a.rope, a.geom.dtype), a.geom.dtype) |
                   ((uint32_t)narrow16(rope_elem(row, ch * 8 + 2 * e + 1, cs, sn, a.rope, a.geom.dtype), a.geom.dtype) << 16);
        *(uint4 *)(a.layer + off) = uint4{w[0], w[1], w[2], w[3]};
        return;
    }
    *(uint4 *)(a.layer + off) = *(const uint4 *)src;
}

} // namespace

template <int G, int GC, bool ROPE> hipError_t launch_flush_g(const AppendArgs &a, hipStream_t s)
{
    const int U = a.batch * a.n_kv_heads;
    constexpr int v_items = G * (kHeadDim / GC) * 2;
    constexpr size_t lds = (size_t)G * kRowPad * sizeof(float) + (size_t)G * kHeadDim + kHeadDim * sizeof(float) +
                           2 * (size_t)(v_items > kThreads ? v_items : kThreads) * sizeof(float);
    const long long items = (long long)a.n_flush_blocks * U * 2;
    if (items > 0x7FFFFFFF) return hipErrorInvalidValue;
    // as many workgroups as the device holds at once (they loop over the items)
    static const int slots = [] {
        int per_cu = 0, dev = 0, cus = 0;
        if (lds > 64 * 1024 &&
            hipFuncSetAttribute((const void *)flush_block_kernel<G, GC, ROPE>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)lds) != hipSuccess)
            return 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, flush_block_kernel<G, GC, ROPE>, kThreads, lds) != hipSuccess ||
            hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
            return 0;
        return per_cu * cus;
    }();
    if (slots < 1) return hipErrorInvalidValue;
    const int grid = items < slots ? (int)items : slots;
    hipLaunchKernelGGL((flush_block_kernel<G, GC, ROPE>), dim3(grid), dim3(kThreads), lds, s, a, (int)items);
    return note_launch(hipGetLastError());
}
template <int G> hipError_t launch_flush_gc(const AppendArgs &a, hipStream_t s)
{
    if (a.rope != 0) {
        if (a.geom.Gc == 32) return launch_flush_g<G, 32, true>(a, s);
        if (a.geom.Gc == 64) return launch_flush_g<G, 64, true>(a, s);
        return launch_flush_g<G, 128, true>(a, s);
    }
    if (a.geom.Gc == 32) return launch_flush_g<G, 32, false>(a, s);
    if (a.geom.Gc == 64) return launch_flush_g<G, 64, false>(a, s);
    return launch_flush_g<G, 128, false>(a, s);
}

template <int GC, int BITS, bool ROPE> hipError_t launch_flush_wave(const AppendArgs &a, hipStream_t s)
{
    const int U = a.batch * a.n_kv_heads;
    const long long items = (long long)a.n_flush_blocks * U * (a.sides ? 1 : 2);
    if (items > 0x7FFFFFFF) return hipErrorInvalidValue;
    static const int slots = [] {
        int per_cu = 0, dev = 0, cus = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, flush_wave_kernel<GC, BITS, ROPE>, kThreads, 0) != hipSuccess ||
            hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
            return 0;
        return per_cu * cus;
    }();
    if (slots < 1) return hipErrorInvalidValue;
    const long long want = (items + kThreads / 64 - 1) / (kThreads / 64);
    const int grid = want < slots ? (int)want : slots;
    hipLaunchKernelGGL((flush_wave_kernel<GC, BITS, ROPE>), dim3(grid), dim3(kThreads), 0, s, a, (int)items);
    return note_launch(hipGetLastError());
}

template <int G, int GC, int BITS, bool ROPE> hipError_t launch_flush_wave_parts(const AppendArgs &a, hipStream_t s)
{
    const int U = a.batch * a.n_kv_heads;
    const long long items = (long long)a.n_flush_blocks * U * 2;
    if (items > 0x7FFFFFFF) return hipErrorInvalidValue;
    constexpr size_t lds = (size_t)(kThreads / 64) * WaveImage<G, GC, BITS, ROPE>::BYTES;
    static const int slots = [] {
        int per_cu = 0, dev = 0, cus = 0;
        if (lds > 64 * 1024 &&
            hipFuncSetAttribute((const void *)flush_wave_parts_kernel<G, GC, BITS, ROPE>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
            return 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, flush_wave_parts_kernel<G, GC, BITS, ROPE>, kThreads, lds) != hipSuccess ||
            hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
            return 0;
        return per_cu * cus;
    }();
    if (slots < 1) return hipErrorInvalidValue;
    const long long want = (items + kThreads / 64 - 1) / (kThreads / 64);
    const int grid = want < slots ? (int)want : slots;
    hipLaunchKernelGGL((flush_wave_parts_kernel<G, GC, BITS, ROPE>), dim3(grid), dim3(kThreads), lds, s, a, (int)items);
    return note_launch(hipGetLastError());
}

template <int G, int GC, int BITS, bool ROPE> hipError_t launch_flush_coop(const AppendArgs &a, hipStream_t s)
{
    const int U = a.batch * a.n_kv_heads;
    const long long items = (long long)a.n_flush_blocks * U * 2;
    if (items > 0x7FFFFFFF) return hipErrorInvalidValue;
    constexpr int threads = 64 * (G / 32);
    static const int slots = [] {
        int per_cu = 0, dev = 0, cus = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, flush_coop_kernel<G, GC, BITS, ROPE>, threads, 0) != hipSuccess ||
            hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
            return 0;
        return (per_cu * cus) & ~1; // even: see the kernel's item order
    }();
    if (slots < 2) return hipErrorInvalidValue;
    const int grid = items < slots ? (int)items : slots; // (items is even)
    hipLaunchKernelGGL((flush_coop_kernel<G, GC, BITS, ROPE>), dim3(grid), dim3(threads), 0, s, a, (int)items);
    return note_launch(hipGetLastError());
}

hipError_t launch_flush(const AppendArgs &a, hipStream_t s)
{
    const int U = a.batch * a.n_kv_heads;
    if (U > 65535) return hipErrorInvalidValue;
    (void)hipGetLastError(); // drop any stale error left by earlier runtime calls of this thread
    const bool wave32 = a.geom.G == 32 && a.geom.k_bits == a.geom.v_bits && a.geom.k_bits != 16;
    if (a.sides != 0 && (!wave32 || a.geom.mean_mode == 1)) return note_launch(hipErrorInvalidValue);
    if (a.geom.mean_mode == 1) {
        if (a.batch > 65535) return hipErrorInvalidValue;
        hipLaunchKernelGGL(xhead_mean_kernel, dim3(a.n_flush_blocks, a.batch, 2), dim3(kThreads), 0, s, a);
        hipError_t e = note_launch(hipGetLastError());
        if (e != hipSuccess) return e;
    }
    const int kb = a.geom.k_bits;
    {
        // blocks of 32 tokens, keys and values of different widths (per-channel mean or none): the keys' side
        // and the values' side as two launches of the one-wavefront-per-item quantiser, each at its own width
        const int vb = a.geom.v_bits, gc = a.geom.Gc;
        const bool widths = (kb == 2 || kb == 4 || kb == 8) && (vb == 2 || vb == 4 || vb == 8) && kb != vb;
        if (a.geom.G == 32 && widths && a.geom.mean_mode != 1 && a.sides == 0 && a.len_dev == nullptr) {
            auto side = [&](int which, int bits, bool rope) -> hipError_t {
                AppendArgs x = a;
                x.sides = which + 1;
                if (!rope) x.rope = 0;
#define TADAKV_SIDE(GCV, R)                                                                       \
    (bits == 2 ? launch_flush_wave<GCV, 2, R>(x, s) : bits == 4 ? launch_flush_wave<GCV, 4, R>(x, s) \
                                                               : launch_flush_wave<GCV, 8, R>(x, s))
                if (rope) return gc == 32 ? TADAKV_SIDE(32, true) : gc == 64 ? TADAKV_SIDE(64, true) : TADAKV_SIDE(128, true);
                return gc == 32 ? TADAKV_SIDE(32, false) : gc == 64 ? TADAKV_SIDE(64, false) : TADAKV_SIDE(128, false);
#undef TADAKV_SIDE
            };
            const hipError_t e = side(0, kb, a.rope != 0);
            if (e != hipSuccess) return e;
            return side(1, vb, false);
        }
    }
    if (a.geom.G == 32 && kb == a.geom.v_bits && kb != 16) {
        // blocks of 32 tokens, one width for keys and values: one wavefront per item, registers only
        const int gc = a.geom.Gc;
#define TADAKV_WAVE(GCV, R)                                                                      \
    (kb == 2 ? launch_flush_wave<GCV, 2, R>(a, s) : kb == 4 ? launch_flush_wave<GCV, 4, R>(a, s) \
                                                           : launch_flush_wave<GCV, 8, R>(a, s))
        if (a.rope != 0) return gc == 32 ? TADAKV_WAVE(32, true) : gc == 64 ? TADAKV_WAVE(64, true) : TADAKV_WAVE(128, true);
        return gc == 32 ? TADAKV_WAVE(32, false) : gc == 64 ? TADAKV_WAVE(64, false) : TADAKV_WAVE(128, false);
#undef TADAKV_WAVE
    }
    // the bulk append of blocks of 64 / 128 tokens: a workgroup per item, one read of the input
    const bool coop = a.len_dev == nullptr && a.sides == 0;
#define TADAKV_COOP(GV, GCV, R) \
    (kb == 2 ? launch_flush_coop<GV, GCV, 2, R>(a, s) : kb == 4 ? launch_flush_coop<GV, GCV, 4, R>(a, s) : launch_flush_coop<GV, GCV, 8, R>(a, s))
    if (coop && a.geom.G == 64 && kb == a.geom.v_bits && kb != 16) {
        if (a.rope != 0) return a.geom.Gc == 32 ? TADAKV_COOP(64, 32, true) : a.geom.Gc == 64 ? TADAKV_COOP(64, 64, true) : TADAKV_COOP(64, 128, true);
        return a.geom.Gc == 32 ? TADAKV_COOP(64, 32, false) : a.geom.Gc == 64 ? TADAKV_COOP(64, 64, false) : TADAKV_COOP(64, 128, false);
    }
    if (coop && a.geom.G == 128 && kb == a.geom.v_bits && kb != 16) {
        if (a.rope != 0) return a.geom.Gc == 32 ? TADAKV_COOP(128, 32, true) : a.geom.Gc == 64 ? TADAKV_COOP(128, 64, true) : TADAKV_COOP(128, 128, true);
        return a.geom.Gc == 32 ? TADAKV_COOP(128, 32, false) : a.geom.Gc == 64 ? TADAKV_COOP(128, 64, false) : TADAKV_COOP(128, 128, false);
    }
#undef TADAKV_COOP
    if (a.geom.G == 64 && kb == a.geom.v_bits && kb != 16) {
        // blocks of 64 tokens: the same arithmetic in two passes over two parts of 32 tokens
        const int gc = a.geom.Gc;
#define TADAKV_PARTS(GV, GCV, R)                                                \
    (kb == 2 ? launch_flush_wave_parts<GV, GCV, 2, R>(a, s)                     \
             : kb == 4 ? launch_flush_wave_parts<GV, GCV, 4, R>(a, s) : launch_flush_wave_parts<GV, GCV, 8, R>(a, s))
        if (a.rope != 0) return gc == 32 ? TADAKV_PARTS(64, 32, true) : gc == 64 ? TADAKV_PARTS(64, 64, true) : TADAKV_PARTS(64, 128, true);
        return gc == 32 ? TADAKV_PARTS(64, 32, false) : gc == 64 ? TADAKV_PARTS(64, 64, false) : TADAKV_PARTS(64, 128, false);
    }
    if (a.geom.G == 128 && a.geom.Gc == 128 && kb == a.geom.v_bits && kb != 16) {
        // blocks of 128 tokens with one value group per token: four parts
        return a.rope != 0 ? TADAKV_PARTS(128, 128, true) : TADAKV_PARTS(128, 128, false);
#undef TADAKV_PARTS
    }
    if (a.geom.G == 32) return launch_flush_gc<32>(a, s);
    if (a.geom.G == 64) return launch_flush_gc<64>(a, s);
    return launch_flush_gc<128>(a, s);
}

bool step_store_supported(const LayerGeom &g)
{
    // the formats of the one-wavefront-per-item quantisers (launch_flush), dense placement
    const bool blocks = g.G == 32 || g.G == 64 || (g.G == 128 && g.Gc == 128);
    return blocks && g.k_bits == g.v_bits && g.k_bits != 16;
}

hipError_t launch_resid_copy(const AppendArgs &a, hipStream_t s)
{
    const int U = a.batch * a.n_kv_heads;
    if (U > 65535) return hipErrorInvalidValue;
    dim3 grid((a.copy_n + 7) / 8, U, 1);
    (void)hipGetLastError(); // drop any stale error left by earlier runtime calls of this thread
    hipLaunchKernelGGL(resid_copy_kernel, grid, dim3(kThreads), 0, s, a);
    return note_launch(hipGetLastError());
}

} // namespace tadakv
