// Dense terms of decode attention under the cross-head mean (arxiv 2506.04642 Eq. 1-2: the mean
// over the heads, one 128-vector per token and per K / V, shared by all kv heads of a sequence).
//
// With K^[h,t,:] = m_K[t,:] + deviation (Eq. 7) the score of query head i against token t is
//   q_i . K^[h,t,:] = q_i . m_K[t,:] + q_i . deviation[h,t,:]
// and with V^ = m_V + deviation (Eq. 8) the output is
//   o_i = sum_t a_t m_V[t,:] + sum_t a_t deviation[h,t,:].
// The deviation terms run on the matrix cores inside the split kernel; the two mean terms are
// plain dense products against a 16-bit stream that every head of the sequence shares:
//   xhead_scores_kernel : xs[b][i][t] = q_i . m_K[b,t,:]            for every packed token, before the split kernel
//   xhead_values_kernel : partial O[u, i, split] += sum_t w_t m_V[b,t,:]   after it, before the merge
// where w_t = p_t 2^(mc - M): p_t is the weight the split kernel wrote relative to its chunk's
// maximum mc, and M the split's final running maximum (both in the exp2 domain).
#include "tadakv_internal.h"
#include <hip/hip_fp16.h>
#include <type_traits>

namespace tadakv {
namespace {

constexpr int kThreads = 256;

__device__ __forceinline__ float widen16(uint16_t v, int dtype)
{
    if (dtype == 1) return __uint_as_float((uint32_t)v << 16);
    return __half2float(__ushort_as_half(v));
}
__device__ __forceinline__ float f16_val(uint16_t h) { return __half2float(__ushort_as_half(h)); }

// mean plane row of (batch b, side which, token t): 128 binary16 values
__device__ __forceinline__ const uint16_t *mean_row(const DecodeArgs &a, int b, int which, int t)
{
    const LayerGeom &gm = a.geom;
    const int lg = 31 - __builtin_clz(gm.G); // G is 32, 64 or 128
    const int blk = t >> lg, tin = t - (blk << lg);
    return (const uint16_t *)(a.layer + gm.xmean_off) + (((long long)b * gm.NB + blk) * 2 + which) * gm.G * kHeadDim +
           tin * kHeadDim;
}

typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));

// grid (ceil(T / 256), batch); a wave takes 64 tokens, 16 at a time.  Scores of 16 query heads
// against 16 tokens over 32 channels are one v_mfma_f32_16x16x32_f16: A = queries (row = head,
// the lane holds channels 8 (l / 16) .. + 7 of the 32), B = the mean rows (column = token, the
// same 8 channels: 16 contiguous bytes of the row), D = [head][token] with lane l holding heads
// 4 (l / 16) .. + 3 of token l % 16.  Queries are narrowed to binary16 (exact for binary16 inputs;
// bfloat16 inputs lose only values below 2^-14 in magnitude).
template <int MT> // 16-head tiles: ceil(Hq / 16)
__global__ __launch_bounds__(kThreads) void xhead_scores_kernel(DecodeArgs a)
{
    const int Hq = a.n_q_heads, b = blockIdx.y;
    const int T = a.n_blocks * a.geom.G;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 15, kg = lane >> 4;
    v8h qa[MT][4];
#pragma unroll
    for (int mt = 0; mt < MT; mt++) {
        const int head = 16 * mt + n;
#pragma unroll
        for (int ks = 0; ks < 4; ks++) {
            uint4 raw = uint4{0u, 0u, 0u, 0u};
            if (head < Hq) raw = *(const uint4 *)(a.q + ((long long)b * Hq + head) * kHeadDim + 32 * ks + 8 * kg);
            const uint32_t wv[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
            for (int e = 0; e < 4; e++) {
                qa[mt][ks][2 * e] = (_Float16)widen16((uint16_t)(wv[e] & 0xFFFFu), a.geom.dtype);
                qa[mt][ks][2 * e + 1] = (_Float16)widen16((uint16_t)(wv[e] >> 16), a.geom.dtype);
            }
        }
    }
    const int t_wave = blockIdx.x * 256 + wave * 64;
    if (t_wave >= T) return;
    // the wave's four tiles of mean rows, all loads in flight at once
    v8h mb[4][4];
#pragma unroll
    for (int tile = 0; tile < 4; tile++) {
        int t = t_wave + 16 * tile + n;
        t = t < T ? t : T - 1; // past the end: any valid row, the result is not stored
        const uint16_t *row = mean_row(a, b, 0, t);
#pragma unroll
        for (int ks = 0; ks < 4; ks++) mb[tile][ks] = *(const v8h *)(row + 32 * ks + 8 * kg);
    }
#pragma unroll
    for (int tile = 0; tile < 4; tile++) {
        const int t = t_wave + 16 * tile + n;
#pragma unroll
        for (int mt = 0; mt < MT; mt++) {
            v4f acc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int ks = 0; ks < 4; ks++) acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(qa[mt][ks], mb[tile][ks], acc, 0, 0, 0);
            if (t < T) {
#pragma unroll
                for (int j = 0; j < 4; j++) {
                    const int head = 16 * mt + 4 * kg + j;
                    if (head < Hq) a.xs[((long long)b * Hq + head) * a.tcap + t] = acc[j];
                }
            }
        }
    }
}

// grid (n_splits, units).  The chunks of a split are the ones the split kernel gave it (chunk
// sp + n_splits j of the unit).  Thread = (channel pair, quarter of the chunk's tokens); every
// thread keeps sums for all query heads of the unit, the four quarters are added at the end.
template <int NI> // query heads per kv head, rounded up to 1, 2, 4 or 8 (weights of the padding heads are zero)
__global__ __launch_bounds__(kThreads) void xhead_values_kernel(DecodeArgs a)
{
    __shared__ float w[kMaxGroupQ][64];
    __shared__ float red[4][kMaxGroupQ][kHeadDim];
    const LayerGeom &gm = a.geom;
    const int sp = blockIdx.x, u = blockIdx.y, ns = a.n_splits, g = a.g;
    const int b = u / a.n_kv_heads, h = u % a.n_kv_heads;
    const int nbc = 64 / gm.G > 0 ? 64 / gm.G : 1;
    const int chunks_total = (a.n_blocks + nbc - 1) / nbc;
    const int T = a.n_blocks * gm.G;
    const int cp = threadIdx.x & 63, tq = threadIdx.x >> 6;
    const int ncap = a.tcap / 64 + 1;
    float acc[NI][2];
#pragma unroll
    for (int i = 0; i < NI; i++) acc[i][0] = acc[i][1] = 0.0f;
    for (int e = threadIdx.x; e < kMaxGroupQ * 64; e += kThreads) w[e >> 6][e & 63] = 0.0f;
    // value plane of this sequence: token t sits (t + (t rounded down to its block)) rows of 128 in
    const uint16_t *vplane = (const uint16_t *)(a.layer + gm.xmean_off) + ((long long)b * gm.NB * 2 + 1) * gm.G * kHeadDim + 2 * cp;
    const int gmask = ~(gm.G - 1);
    // weight staging: thread e handles (head e / 64, token e % 64) of the chunk, twice if g > 4
    const int wi = threadIdx.x >> 6, wt_tok = threadIdx.x & 63;
    float Msp[2];
    long long wq[2];
#pragma unroll
    for (int r = 0; r < 2; r++) {
        const int i = wi + 4 * r < g ? wi + 4 * r : 0;
        Msp[r] = a.ws[((long long)(u * g + i) * ns + sp) * kPartialStride + kHeadDim];
        wq[r] = (long long)b * a.n_q_heads + h * g + i;
    }
    // Two chunks ahead: the weights of this thread's (head, token) entries and its 16 mean words of
    // a chunk are loaded into a register slot two iterations before they are used.
    uint32_t mv[2][16];
    float xpv[2][2], xmv[2][2];
    auto fetch = [&](auto slot_c, int c) {
        constexpr int slot = decltype(slot_c)::value;
#pragma unroll
        for (int r = 0; r < 2; r++) {
            const int t = c * 64 + wt_tok;
            xpv[slot][r] = t < T ? a.xp[wq[r] * a.tcap + t] : 0.0f;
            xmv[slot][r] = a.xmc[wq[r] * ncap + c];
        }
#pragma unroll
        for (int k = 0; k < 16; k++) {
            const int t = c * 64 + 4 * k + tq;
            mv[slot][k] = t < T ? *(const uint32_t *)(vplane + (long long)(t + (t & gmask)) * kHeadDim) : 0u;
        }
    };
    auto step = [&](auto slot_c, int c_next) {
        constexpr int slot = decltype(slot_c)::value;
        __syncthreads(); // the previous chunk's weights have been used
#pragma unroll
        for (int r = 0; r < 2; r++) {
            const int i = wi + 4 * r;
            if (i < g) w[i][wt_tok] = xpv[slot][r] * exp2f(xmv[slot][r] - Msp[r]);
        }
        uint32_t cur[16];
#pragma unroll
        for (int k = 0; k < 16; k++) cur[k] = mv[slot][k];
        if (c_next < chunks_total) fetch(slot_c, c_next);
        __syncthreads();
#pragma unroll
        for (int k = 0; k < 16; k++) {
            const float m0 = f16_val((uint16_t)(cur[k] & 0xFFFFu)), m1 = f16_val((uint16_t)(cur[k] >> 16));
#pragma unroll
            for (int i = 0; i < NI; i++) {
                const float wt = w[i][4 * k + tq];
                acc[i][0] += wt * m0;
                acc[i][1] += wt * m1;
            }
        }
    };
    const std::integral_constant<int, 0> s0;
    const std::integral_constant<int, 1> s1;
    if (sp < chunks_total) fetch(s0, sp);
    if (sp + ns < chunks_total) fetch(s1, sp + ns);
    for (int c = sp; c < chunks_total; c += 2 * ns) {
        step(s0, c + 2 * ns);
        if (c + ns < chunks_total) step(s1, c + 3 * ns);
    }
#pragma unroll
    for (int i = 0; i < NI; i++) {
        red[tq][i][2 * cp] = acc[i][0];
        red[tq][i][2 * cp + 1] = acc[i][1];
    }
    __syncthreads();
    for (int e = threadIdx.x; e < g * kHeadDim; e += kThreads) {
        const int i = e >> 7, ch = e & 127;
        const float sum = (red[0][i][ch] + red[1][i][ch]) + (red[2][i][ch] + red[3][i][ch]);
        a.ws[((long long)(u * g + i) * ns + sp) * kPartialStride + ch] += sum;
    }
}

} // namespace

hipError_t launch_xhead_scores(const DecodeArgs &a, hipStream_t s)
{
    const int T = a.n_blocks * a.geom.G;
    if (T == 0) return hipSuccess;
    if (a.batch > 65535 || a.n_q_heads > 64) return hipErrorInvalidValue;
    dim3 grid((T + 255) / 256, a.batch);
    const int mt = (a.n_q_heads + 15) / 16;
    (void)hipGetLastError(); // drop any stale error left by earlier runtime calls of this thread
    if (mt <= 1) hipLaunchKernelGGL(xhead_scores_kernel<1>, grid, dim3(kThreads), 0, s, a);
    else if (mt <= 2) hipLaunchKernelGGL(xhead_scores_kernel<2>, grid, dim3(kThreads), 0, s, a);
    else hipLaunchKernelGGL(xhead_scores_kernel<4>, grid, dim3(kThreads), 0, s, a);
    return note_launch(hipGetLastError());
}

hipError_t launch_xhead_values(const DecodeArgs &a, hipStream_t s)
{
    if (a.n_blocks == 0) return hipSuccess;
    if (a.batch * a.n_kv_heads > 65535) return hipErrorInvalidValue;
    dim3 grid(a.n_splits, a.batch * a.n_kv_heads);
    (void)hipGetLastError(); // drop any stale error left by earlier runtime calls of this thread
    if (a.g <= 1) hipLaunchKernelGGL(xhead_values_kernel<1>, grid, dim3(kThreads), 0, s, a);
    else if (a.g <= 2) hipLaunchKernelGGL(xhead_values_kernel<2>, grid, dim3(kThreads), 0, s, a);
    else if (a.g <= 4) hipLaunchKernelGGL(xhead_values_kernel<4>, grid, dim3(kThreads), 0, s, a);
    else hipLaunchKernelGGL(xhead_values_kernel<8>, grid, dim3(kThreads), 0, s, a);
    return note_launch(hipGetLastError());
}

} // namespace tadakv
