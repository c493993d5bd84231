// Decode attention over the packed cache, portable vector-ALU version (gfx950), and the
// cross-split merge.
//
// One workgroup handles one (sequence, kv head) and one contiguous range of blocks ("split") and
// serves all g = Hq/Hkv query heads of that kv head.  Per block it evaluates, without ever
// materialising the reconstructed keys and values (arxiv 2506.04642 Eq. 5-8):
//   score_t = ( sum_c (q_c s_c) code_tc + sum_c q_c (z_c + m_c) ) / sqrt(d)         keys, Eq. 5, 7
//   o_c     = sum_t (p_t s_tg) code_tc + sum_t p_t z_tg + m_c sum_t p_t             values, Eq. 6, 8
// with an online softmax across blocks (flash decoding, App. A).  Raw residual tokens (Sec. 3.3,
// Eq. 9-10) and 16-bit layers go through the same code with scale 1, zero 0.
// The split's running (max, sum, output) goes to the workspace; merge_kernel combines the splits
// with the log-sum-exp identity, in a fixed order (no atomics), so results are reproducible.
#include "tadakv_internal.h"
#include <hip/hip_fp16.h>

namespace tadakv {
namespace {

constexpr int kThreads = 256;
constexpr float kLog2e = 1.4426950408889634f;

__device__ __forceinline__ float widen16(uint16_t v, int dtype)
{
    if (dtype == 1) return __uint_as_float((uint32_t)v << 16);
    return __half2float(__ushort_as_half(v));
}
__device__ __forceinline__ float f16_val(uint16_t h) { return __half2float(__ushort_as_half(h)); }
// binary32 -> the 16-bit type, round to nearest even (finite inputs)
__device__ __forceinline__ uint16_t narrow16_rne(float f, int dtype)
{
    if (dtype == 1) {
        const uint32_t u = __float_as_uint(f);
        return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
    }
    return __half_as_ushort(__float2half_rn(f));
}

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// index of the 32-bit word that holds key codes (t, c0 .. c0 + 32/B - 1)
template <int B> __device__ __forceinline__ int k_word(int t, int c0)
{
    const int tt = t >> 4, n = t & 15, cg = c0 >> 4;
    if (B == 8) return ((((tt * 2 + (cg & 1)) * 4 + (cg >> 1)) * 16 + n) << 2) + ((c0 & 15) >> 2);
    if (B == 4) return (((tt * 4 + (cg >> 1)) * 16 + n) << 2) + (cg & 1) * 2 + ((c0 & 15) >> 3);
    if (B == 2) return ((((tt >> 1) * 4 + (cg >> 1)) * 16 + n) << 2) + (tt & 1) * 2 + (cg & 1);
    return t * 64 + (c0 >> 1); // raw 16-bit rows
}
// index of the word that holds value codes (t0 .. t0 + 32/B - 1, c)
template <int B> __device__ __forceinline__ int v_word(int t0, int c, int nt)
{
    const int tt = t0 >> 4, ct = c >> 4, n = c & 15;
    if (B == 8) return (((ct * nt + tt) * 16 + n) << 2) + ((t0 & 15) >> 2);
    if (B == 4) return ((((ct >> 1) * nt + tt) * 16 + n) << 2) + (ct & 1) * 2 + ((t0 & 15) >> 3);
    return ((((ct >> 2) * nt + tt) * 16 + n) << 2) + (ct & 3);
}

struct Smem {
    float *qf, *qs, *part, *ps, *pz, *psum, *alpha, *mrun, *lrun, *bpart, *vmean, *pp;
    uint32_t *kc, *vc, *vmeta;
    uint16_t *xk, *xv; // cross-head mean tiles [G][128] of the block (keys, values)
};

// One block (or one chunk of raw tokens) of one unit.  KB/VB = 16 means raw rows.
template <int KB, int VB>
__device__ __forceinline__ void process_block(const DecodeArgs &a, const Smem &sm, int ntok,
                                              const unsigned char *kcodes, const unsigned char *kscale,
                                              const unsigned char *kzero, const unsigned char *kmean,
                                              const unsigned char *vcodes, const unsigned char *vmeta,
                                              const unsigned char *vmean, const unsigned char *xmean_k,
                                              const unsigned char *xmean_v, float (&acc)[kMaxGroupQ / 2])
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = a.g;
    const int G = (KB == 16) ? 32 : a.geom.G;     // row stride of the LDS score arrays
    const int ng = (VB == 16) ? 1 : kHeadDim / a.geom.Gc;
    const int nt = a.geom.G >> 4;

    __syncthreads(); // the previous block's readers are done with the staging buffers

    // ---- stage codes and value metadata
    {
        const int kbytes = (KB == 16) ? ntok * 256 : a.geom.G * kHeadDim * KB / 8;
        for (int i = tid; i < kbytes / 16; i += kThreads) ((uint4 *)sm.kc)[i] = ((const uint4 *)kcodes)[i];
        const int vbytes = (VB == 16) ? ntok * 256 : a.geom.G * kHeadDim * VB / 8;
        for (int i = tid; i < vbytes / 16; i += kThreads) ((uint4 *)sm.vc)[i] = ((const uint4 *)vcodes)[i];
        if (xmean_k) {
            // cross-head mean (Eq. 1-2): one binary16 row per token, shared by all kv heads
            for (int i = tid; i < a.geom.G * 16; i += kThreads) {
                ((uint4 *)sm.xk)[i] = ((const uint4 *)xmean_k)[i];
                ((uint4 *)sm.xv)[i] = ((const uint4 *)xmean_v)[i];
            }
        }
        if (VB != 16) {
            for (int i = tid; i < a.geom.G * ng; i += kThreads) sm.vmeta[i] = ((const uint32_t *)vmeta)[i];
            if (tid < kHeadDim) sm.vmean[tid] = vmean ? f16_val(((const uint16_t *)vmean)[tid]) : 0.0f;
        }
    }
    // ---- fold the key scale into q, and the zero / mean terms into one number per head
    {
        const int c = tid & 127, hsel = tid >> 7;
        float s = 1.0f, zm = 0.0f;
        if (KB != 16) {
            s = f16_val(((const uint16_t *)kscale)[c]);
            zm = f16_val(((const uint16_t *)kzero)[c]);
            if (kmean) zm += f16_val(((const uint16_t *)kmean)[c]);
        }
        for (int i = hsel; i < g; i += 2) {
            const float qv = sm.qf[i * kHeadDim + c];
            sm.qs[i * kHeadDim + c] = qv * s;
            const float bsum = wave_sum(qv * zm);
            if (lane == 0) sm.bpart[i * 2 + (wave & 1)] = bsum;
        }
    }
    __syncthreads();

    // ---- scores: each work item is (token, head, channel half)
    for (int idx = tid; idx < ntok * g * 2; idx += kThreads) {
        const int t = idx % ntok, rest = idx / ntok;
        const int i = rest % g, half = rest / g;
        const float *qrow = sm.qs + i * kHeadDim;
        float s = 0.0f;
        constexpr int per = (KB == 16) ? 2 : 32 / KB;
        for (int c0 = half * 64; c0 < half * 64 + 64; c0 += per) {
            const uint32_t w = sm.kc[k_word<KB>(t, c0)];
            if (KB == 16) {
                s += qrow[c0] * widen16((uint16_t)(w & 0xFFFFu), a.geom.dtype);
                s += qrow[c0 + 1] * widen16((uint16_t)(w >> 16), a.geom.dtype);
            } else {
#pragma unroll
                for (int e = 0; e < per; e++)
                    s += qrow[c0 + e] *
                         (float)((w >> (8 * (e & 3) + (KB & 15) * (e >> 2))) & ((1u << (KB & 15)) - 1u));
            }
        }
        if (KB != 16 && xmean_k) {
            const float *qraw = sm.qf + i * kHeadDim;
            const uint16_t *mrow = sm.xk + t * kHeadDim;
            for (int c = half * 64; c < half * 64 + 64; c++) s += qraw[c] * f16_val(mrow[c]);
        }
        sm.part[(half * g + i) * G + t] = s;
    }
    __syncthreads();

    // ---- online softmax: wave w owns heads w, w+4
    const float sc_scale = 0.08838834764831845f * kLog2e; // 1/sqrt(128) in the exp2 domain
    for (int i = wave; i < g; i += 4) {
        const float beta = sm.bpart[i * 2] + sm.bpart[i * 2 + 1];
        float sv[2];
        float bmax = -INFINITY;
#pragma unroll
        for (int k = 0; k < 2; k++) {
            const int t = lane + 64 * k;
            sv[k] = -INFINITY;
            if (t < ntok) sv[k] = (sm.part[i * G + t] + sm.part[(g + i) * G + t] + beta) * sc_scale;
            bmax = fmaxf(bmax, sv[k]);
        }
        bmax = wave_max(bmax);
        const float m_old = sm.mrun[i];
        const float m_new = fmaxf(m_old, bmax);
        const float alpha = exp2f(m_old - m_new);
        float psum = 0.0f;
        float pz[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int k = 0; k < 2; k++) {
            const int t = lane + 64 * k;
            if (t < ntok) {
                const float p = exp2f(sv[k] - m_new);
                psum += p;
                sm.pp[i * G + t] = p;
                if (VB == 16) {
                    sm.ps[i * G + t] = p;
                } else {
                    for (int gam = 0; gam < ng; gam++) {
                        const uint32_t mz = sm.vmeta[t * ng + gam];
                        sm.ps[(i * G + t) * ng + gam] = p * f16_val((uint16_t)(mz & 0xFFFFu));
                        pz[gam] += p * f16_val((uint16_t)(mz >> 16));
                    }
                }
            }
        }
        psum = wave_sum(psum);
        if (VB != 16)
            for (int gam = 0; gam < ng; gam++) pz[gam] = wave_sum(pz[gam]);
        if (lane == 0) {
            sm.alpha[i] = alpha;
            sm.mrun[i] = m_new;
            sm.lrun[i] = sm.lrun[i] * alpha + psum;
            sm.psum[i] = psum;
            for (int gam = 0; gam < ng; gam++) sm.pz[i * 4 + gam] = pz[gam];
        }
    }
    __syncthreads();

    // ---- output: thread owns channel c for heads hsel, hsel+2, ...
    {
        const int c = tid & 127, hsel = tid >> 7;
        const int gam = (VB == 16) ? 0 : c / a.geom.Gc;
        float add[kMaxGroupQ / 2];
#pragma unroll
        for (int k = 0; k < kMaxGroupQ / 2; k++) add[k] = 0.0f;
        if (VB == 16) {
            const uint16_t *vr = (const uint16_t *)sm.vc;
            for (int t = 0; t < ntok; t++) {
                const float v = widen16(vr[t * kHeadDim + c], a.geom.dtype);
#pragma unroll
                for (int k = 0; k < kMaxGroupQ / 2; k++) {
                    const int i = hsel + 2 * k;
                    if (i < g) add[k] += sm.ps[i * G + t] * v;
                }
            }
        } else {
            constexpr int per = 32 / (VB & 15 ? VB & 15 : 16);
            for (int t0 = 0; t0 < ntok; t0 += per) {
                const uint32_t w = sm.vc[v_word<VB == 16 ? 8 : VB>(t0, c, nt)];
#pragma unroll
                for (int e = 0; e < per; e++) {
                    const float code =
                        (float)((w >> (8 * (e & 3) + (VB & 15) * (e >> 2))) & ((1u << (VB & 15)) - 1u));
#pragma unroll
                    for (int k = 0; k < kMaxGroupQ / 2; k++) {
                        const int i = hsel + 2 * k;
                        if (i < g) add[k] += sm.ps[(i * G + t0 + e) * ng + gam] * code;
                    }
                }
            }
        }
        if (VB != 16 && xmean_v) {
            for (int t = 0; t < ntok; t++) {
                const float mv = f16_val(sm.xv[t * kHeadDim + c]);
#pragma unroll
                for (int k = 0; k < kMaxGroupQ / 2; k++) {
                    const int i = hsel + 2 * k;
                    if (i < g) add[k] += sm.pp[i * G + t] * mv;
                }
            }
        }
#pragma unroll
        for (int k = 0; k < kMaxGroupQ / 2; k++) {
            const int i = hsel + 2 * k;
            if (i < g) {
                float extra = 0.0f;
                if (VB != 16) extra = sm.pz[i * 4 + gam] + sm.vmean[c] * sm.psum[i];
                acc[k] = acc[k] * sm.alpha[i] + add[k] + extra;
            }
        }
    }
}

template <int KB, int VB> __global__ __launch_bounds__(kThreads) void decode_split_valu_kernel(DecodeArgs a)
{
    extern __shared__ float lds[];
    const LayerGeom &gm = a.geom;
    const int g = a.g, G = gm.G;
    Smem sm;
    float *p = lds;
    sm.qf = p;     p += kMaxGroupQ * kHeadDim;
    sm.qs = p;     p += kMaxGroupQ * kHeadDim;
    sm.part = p;   p += 2 * g * G;
    sm.ps = p;     p += g * G * 4;
    sm.pz = p;     p += kMaxGroupQ * 4;
    sm.psum = p;   p += kMaxGroupQ;
    sm.alpha = p;  p += kMaxGroupQ;
    sm.mrun = p;   p += kMaxGroupQ;
    sm.lrun = p;   p += kMaxGroupQ;
    sm.bpart = p;  p += kMaxGroupQ * 2;
    sm.vmean = p;  p += kHeadDim;
    sm.pp = p;     p += g * G;
    sm.vmeta = (uint32_t *)p; p += G * 4;
    // staging sized for the widest case: 8-bit codes of a block, or 32 raw 16-bit rows
    const int code_words = G * kHeadDim * 8 / 32 > 32 * 64 ? G * kHeadDim * 8 / 32 : 32 * 64;
    sm.kc = (uint32_t *)p; p += code_words;
    sm.vc = (uint32_t *)p; p += code_words;
    sm.xk = (uint16_t *)p; p += (gm.mean_mode == 1 ? G * kHeadDim / 2 : 0);
    sm.xv = (uint16_t *)p;

    const int sp = blockIdx.x, u = blockIdx.y;
    const int b = u / a.n_kv_heads, h = u % a.n_kv_heads;
    const int tid = threadIdx.x;

    // q of this kv head's g query heads, widened
    for (int i = tid; i < g * kHeadDim; i += kThreads)
        sm.qf[i] = widen16(a.q[((long long)b * a.n_q_heads + h * g) * kHeadDim + i], gm.dtype);
    if (tid < kMaxGroupQ) {
        sm.mrun[tid] = -INFINITY;
        sm.lrun[tid] = 0.0f;
    }
    float acc[kMaxGroupQ / 2];
#pragma unroll
    for (int k = 0; k < kMaxGroupQ / 2; k++) acc[k] = 0.0f;

    const int nb_seq = seq_blocks(a, b), r_seq = seq_resid(a, b); // this sequence's packed blocks and raw tokens
    const int work = nb_seq + (r_seq > 0 ? 1 : 0);
    const int w0 = sp * a.blocks_per_split;
    int w1 = w0 + a.blocks_per_split;
    if (w1 > work) w1 = work;
    const int b_end = w1 < nb_seq ? w1 : nb_seq;

    for (int j = w0; j < b_end; j++) {
        const unsigned char *rec = a.layer + record_offset(gm, a.n_kv_heads, b, u % a.n_kv_heads, j);
        if (KB == 16) {
            for (int t0 = 0; t0 < G; t0 += 32)
                process_block<16, 16>(a, sm, 32, rec + gm.k_codes + t0 * 256, nullptr, nullptr, nullptr,
                                      rec + gm.v_codes + t0 * 256, nullptr, nullptr, nullptr, nullptr, acc);
        } else {
            const unsigned char *xm = gm.mean_mode == 1
                                          ? a.layer + xmean_offset(gm, b, j, 0)
                                          : nullptr;
            process_block<KB, VB>(a, sm, G, rec + gm.k_codes, rec + gm.k_scale, rec + gm.k_zero,
                                  gm.k_mean >= 0 ? rec + gm.k_mean : nullptr, rec + gm.v_codes,
                                  rec + gm.v_meta, gm.v_mean >= 0 ? rec + gm.v_mean : nullptr, xm,
                                  xm ? xm + G * kHeadDim * 2 : nullptr, acc);
        }
    }
    if (w0 < w1 && w1 > nb_seq && r_seq > 0) {
        const unsigned char *kr = a.layer + gm.k_resid_off + (long long)u * gm.R * 256;
        const unsigned char *vr = a.layer + gm.v_resid_off + (long long)u * gm.R * 256;
        for (int t0 = 0; t0 < r_seq; t0 += 32) {
            const int n = r_seq - t0 < 32 ? r_seq - t0 : 32;
            process_block<16, 16>(a, sm, n, kr + t0 * 256, nullptr, nullptr, nullptr, vr + t0 * 256,
                                  nullptr, nullptr, nullptr, nullptr, acc);
        }
    }
    __syncthreads();

    // partial result of this split
    const int c = tid & 127, hsel = tid >> 7;
#pragma unroll
    for (int k = 0; k < kMaxGroupQ / 2; k++) {
        const int i = hsel + 2 * k;
        if (i < g) {
            float *dst = a.ws + (((long long)u * g + i) * a.n_splits + sp) * kPartialStride;
            dst[c] = acc[k];
            if (c == 0) {
                dst[kHeadDim] = sm.mrun[i];
                dst[kHeadDim + 1] = sm.lrun[i];
            }
        }
    }
}

// Cross-split merge (flash decoding, App. A):
//   out[b, head] = sum_j o_j 2^(m_j - M) / sum_j l_j 2^(m_j - M),  M = max_j m_j.
// One workgroup per query head, a lane owns two channels; wave w adds up the
// splits w, w + 4, ... in rising order and the four sums are added in wave order, so the result
// does not depend on timing.  A long-context launch has a hundred splits per head and few heads:
// the loads of a wave are independent and issued several splits at a time.
__global__ __launch_bounds__(256) void merge_kernel(DecodeArgs a)
{
    __shared__ float red[4][3][64];
    __shared__ float mx[4];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int uq = blockIdx.x; // (unit, head-in-group)
    const int u = uq / a.g, i = uq % a.g;
    const int ns = a.n_splits;
    const float *base = a.ws + (long long)uq * ns * kPartialStride;
    float M = -INFINITY;
    for (int j = threadIdx.x; j < ns; j += 256) M = fmaxf(M, base[j * kPartialStride + kHeadDim]);
    M = wave_max(M);
    if (lane == 0) mx[wave] = M;
    __syncthreads();
    M = fmaxf(fmaxf(mx[0], mx[1]), fmaxf(mx[2], mx[3]));
    float n0 = 0.0f, n1 = 0.0f, den = 0.0f;
#pragma unroll 8
    for (int j = wave; j < ns; j += 4) {
        const float *pj = base + j * kPartialStride;
        const float w = pj[kHeadDim] == -INFINITY ? 0.0f : exp2f(pj[kHeadDim] - M);
        const float2 o = *(const float2 *)(pj + 2 * lane);
        n0 += o.x * w;
        n1 += o.y * w;
        den += pj[kHeadDim + 1] * w;
    }
    // cross-head mean: the value mean plane's share, already relative to M (one term per range)
    if (a.xo && a.n_blocks > 0) {
        const float *xb = a.xo + (long long)uq * a.n_xr * kHeadDim;
#pragma unroll 8
        for (int r = wave; r < a.n_xr; r += 4) {
            const float2 o = *(const float2 *)(xb + r * kHeadDim + 2 * lane);
            n0 += o.x;
            n1 += o.y;
        }
    }
    red[wave][0][lane] = n0;
    red[wave][1][lane] = n1;
    red[wave][2][lane] = den;
    __syncthreads();
    if (wave != 0) return;
    n0 = ((red[0][0][lane] + red[1][0][lane]) + red[2][0][lane]) + red[3][0][lane];
    n1 = ((red[0][1][lane] + red[1][1][lane]) + red[2][1][lane]) + red[3][1][lane];
    den = ((red[0][2][lane] + red[1][2][lane]) + red[2][2][lane]) + red[3][2][lane];
    const int b = u / a.n_kv_heads, h = u % a.n_kv_heads;
    float2 r;
    // a sequence that holds no token (every split empty, M == -inf) gives zeros
    r.x = M == -INFINITY ? 0.0f : n0 / den;
    r.y = M == -INFINITY ? 0.0f : n1 / den;
    const long long o = ((long long)b * a.n_q_heads + h * a.g + i) * kHeadDim + 2 * lane;
    if (a.out16) *(uint32_t *)(a.out16 + o) = (uint32_t)narrow16_rne(r.x, a.geom.dtype) | ((uint32_t)narrow16_rne(r.y, a.geom.dtype) << 16);
    else *(float2 *)(a.out + o) = r;
    // a decode step on device-resident lengths ends here: the state after the step becomes the current
    // one (no workgroup of this kernel reads the lengths)
    if (a.len_dev && blockIdx.x == 0 && lane == 0) a.len_dev[4 * a.batch] = (a.len_dev[4 * a.batch] & 1) ^ 1;
}

// code (token t, channel c) of a block's key (which = 0) or value side, from the packed words
template <int B> __device__ __forceinline__ uint32_t code_of(const unsigned char *codes, int which, int G, int t, int c)
{
    constexpr int PW = 32 / B; // codes per word
    const uint32_t *w = (const uint32_t *)codes;
    int j; // number of the code inside its word: code 4 f + y is field f of byte y
    uint32_t word;
    if (which == 0) {
        word = w[k_word<B>(t, c - c % PW)];
        j = c % PW;
    } else {
        word = w[v_word<B>(t - t % PW, c, G / 16)];
        j = t % PW;
    }
    return (word >> (B * (j >> 2) + 8 * (j & 3))) & ((1u << B) - 1u);
}

// Reconstruction (Eq. 7-8): x^ = mean + (zero + scale * code) in binary32, one rounding per
// operation, in that order; raw rows (16-bit layers, the residual buffer) are widened.
// grid (blocks of the longest sequence + 1, units, K | V): workgroup (j, u, which) writes block j of
// unit u, the last index of x the unit's raw tail.  out [batch][t_cap][n_kv_heads][128] binary32.
__global__ __launch_bounds__(kThreads) void dequant_kernel(DequantArgs q)
{
    const DecodeArgs &a = q.d;
    const LayerGeom &gm = a.geom;
    const int G = gm.G, u = blockIdx.y, which = blockIdx.z;
    const int b = u / a.n_kv_heads, h = u % a.n_kv_heads;
    float *out = which == 0 ? q.k_out : q.v_out;
    if (!out) return;
    const int nb = seq_blocks(a, b), r = seq_resid(a, b);
    const int bits = which == 0 ? gm.k_bits : gm.v_bits;
    float *dst_u = out + ((long long)b * q.t_cap * a.n_kv_heads + h) * kHeadDim; // token stride: n_kv_heads * 128
    const long long tstride = (long long)a.n_kv_heads * kHeadDim;
    if ((int)blockIdx.x == a.n_blocks) {
        const unsigned char *raw = a.layer + (which == 0 ? gm.k_resid_off : gm.v_resid_off) + (long long)u * gm.R * 256;
        for (int e = threadIdx.x; e < r * kHeadDim; e += kThreads) {
            const int t = e / kHeadDim, c = e % kHeadDim;
            dst_u[(long long)(nb * G + t) * tstride + c] = widen16(*(const uint16_t *)(raw + t * 256 + c * 2), gm.dtype);
        }
        return;
    }
    const int j = blockIdx.x;
    if (j >= nb) return;
    const unsigned char *rec = a.layer + record_offset(gm, a.n_kv_heads, b, h, j);
    const unsigned char *codes = rec + (which == 0 ? gm.k_codes : gm.v_codes);
    const uint16_t *xm = gm.mean_mode == 1 && bits != 16 ? (const uint16_t *)(a.layer + xmean_offset(gm, b, j, which)) : nullptr;
    const int ng = kHeadDim / gm.Gc;
    for (int e = threadIdx.x; e < G * kHeadDim; e += kThreads) {
        const int t = e / kHeadDim, c = e % kHeadDim;
        float x;
        if (bits == 16) {
            x = widen16(*(const uint16_t *)(codes + (t * kHeadDim + c) * 2), gm.dtype);
        } else {
            const uint32_t code = bits == 2 ? code_of<2>(codes, which, G, t, c)
                                            : bits == 4 ? code_of<4>(codes, which, G, t, c) : code_of<8>(codes, which, G, t, c);
            float sc, z, m = 0.0f;
            if (which == 0) {
                sc = f16_val(*(const uint16_t *)(rec + gm.k_scale + c * 2));
                z = f16_val(*(const uint16_t *)(rec + gm.k_zero + c * 2));
                if (gm.k_mean >= 0) m = f16_val(*(const uint16_t *)(rec + gm.k_mean + c * 2));
            } else {
                const uint32_t sz = *(const uint32_t *)(rec + gm.v_meta + (t * ng + c / gm.Gc) * 4);
                sc = f16_val((uint16_t)(sz & 0xFFFFu));
                z = f16_val((uint16_t)(sz >> 16));
                if (gm.v_mean >= 0) m = f16_val(*(const uint16_t *)(rec + gm.v_mean + c * 2));
            }
            if (xm) m = f16_val(xm[t * kHeadDim + c]);
            x = __fadd_rn(m, __fadd_rn(z, __fmul_rn(sc, (float)code)));
        }
        dst_u[(long long)(j * G + t) * tstride + c] = x;
    }
}

template <int KB, int VB> hipError_t launch_one(const DecodeArgs &a, hipStream_t s)
{
    const int g = a.g, G = a.geom.G;
    size_t floats = 2 * kMaxGroupQ * kHeadDim + 2 * g * G + g * G * 4 + kMaxGroupQ * 4 + 4 * kMaxGroupQ +
                    kMaxGroupQ * 2 + kHeadDim + g * G + G * 4;
    if (a.geom.mean_mode == 1) floats += G * kHeadDim; // two binary16 mean tiles
    const size_t code_words = (size_t)G * kHeadDim * 8 / 32 > 32 * 64 ? (size_t)G * kHeadDim * 8 / 32 : 32 * 64;
    const size_t lds = (floats + 2 * code_words) * 4;
    static size_t granted = 0;
    if (lds > 64 * 1024 && lds > granted) {
        hipError_t e = hipFuncSetAttribute((const void *)decode_split_valu_kernel<KB, VB>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        granted = lds;
    }
    dim3 grid(a.n_splits, a.batch * a.n_kv_heads);
    (void)hipGetLastError(); // drop any stale error left by earlier runtime calls of this thread
    hipLaunchKernelGGL((decode_split_valu_kernel<KB, VB>), grid, dim3(kThreads), lds, s, a);
    return note_launch(hipGetLastError());
}

} // namespace

hipError_t launch_decode_split_valu(const DecodeArgs &a, hipStream_t s)
{
    if (a.batch * a.n_kv_heads > 65535) return hipErrorInvalidValue;
    const int kb = a.geom.k_bits, vb = a.geom.v_bits;
    if ((kb == 16) != (vb == 16)) return hipErrorInvalidValue; // mixed raw / packed sides: not built
    if (kb == 16) return launch_one<16, 16>(a, s);
#define TADAKV_CASE(K_, V_) if (kb == K_ && vb == V_) return launch_one<K_, V_>(a, s);
    TADAKV_CASE(2, 2) TADAKV_CASE(2, 4) TADAKV_CASE(2, 8)
    TADAKV_CASE(4, 2) TADAKV_CASE(4, 4) TADAKV_CASE(4, 8)
    TADAKV_CASE(8, 2) TADAKV_CASE(8, 4) TADAKV_CASE(8, 8)
#undef TADAKV_CASE
    return hipErrorInvalidValue;
}

hipError_t launch_dequant(const DequantArgs &q, hipStream_t s)
{
    const DecodeArgs &a = q.d;
    const int U = a.batch * a.n_kv_heads;
    if (U > 65535) return hipErrorInvalidValue;
    (void)hipGetLastError(); // drop any stale error left by earlier runtime calls of this thread
    hipLaunchKernelGGL(dequant_kernel, dim3(a.n_blocks + 1, U, 2), dim3(kThreads), 0, s, q);
    return note_launch(hipGetLastError());
}

hipError_t launch_decode_merge(const DecodeArgs &a, hipStream_t s)
{
    dim3 grid(a.batch * a.n_q_heads);
    (void)hipGetLastError(); // drop any stale error left by earlier runtime calls of this thread
    hipLaunchKernelGGL(merge_kernel, grid, dim3(256), 0, s, a);
    return note_launch(hipGetLastError());
}

} // namespace tadakv
