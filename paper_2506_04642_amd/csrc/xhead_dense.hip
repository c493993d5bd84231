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
//   xhead_values_kernel : xo[b][i][range] = sum_{t in range} w_t m_V[b,t,:]   after it, before the merge
// where w_t = p_t 2^(mc - M): p_t is the weight the split kernel wrote relative to its chunk's
// maximum mc, and M the largest of the head's split maxima (both in the exp2 domain).
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

// mean plane row of (batch b, side which, token t): 128 binary16 values
__device__ __forceinline__ const uint16_t *mean_row(const DecodeArgs &a, int b, int which, int t)
{
    const LayerGeom &gm = a.geom;
    const int lg = 31 - __builtin_clz(gm.G); // G is 32, 64 or 128
    const int blk = t >> lg, tin = t - (blk << lg);
    return (const uint16_t *)(a.layer + xmean_offset(gm, b, blk, which)) + tin * kHeadDim;
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
    const int T = seq_blocks(a, b) * a.geom.G;
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

// One workgroup per (sequence, range of 64-token chunks), all query heads of the sequence at once:
// the value mean plane is shared by the sequence's kv heads, so its rows are read once.  Per
// chunk the workgroup puts the 64 value-mean rows and the weights of the query heads (as a
// binary16 pair hi + lo, so that nothing is lost) in LDS; wave v then owns channels
// 32 v .. 32 v + 31 and accumulates
//   D[head][channel] += W[head][token] . M[token][channel]
// with v_mfma_f32_16x16x32_f16 (A = weights: row = head, 8 consecutive tokens per lane; B = mean:
// column = channel, the same 8 tokens gathered from 8 rows of the LDS tile).  The weights are
// brought to the head's largest split maximum M (the one the merge uses):
//   w_t = p_t 2^(mc - M),  p_t relative to the chunk maximum mc as the split kernel wrote it,
// so the result needs no further factor and the merge adds it to its numerator.
// (Tried: waves that stage their own 64 x 32 slab and never meet at a barrier -- a row per lane
// makes every load instruction touch 64 cache lines, and the kernel ran at half the speed.  One
// workgroup per (kv head, split): the plane went through L2 once per kv head, 127 us per layer
// on the full-cache workload.)
constexpr int kMvStride = 132; // halfs per LDS row of the mean tile: rows 8 apart start in different banks
constexpr int kWStride = 72;   // halfs per LDS row of the weights

template <int MT> // 16-head tiles: ceil(Hq / 16)
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(MT <= 2 ? 3 : 1, 8))) void xhead_values_kernel(DecodeArgs a)
{
    constexpr int NR = 4 * MT; // heads per thread in the weight staging
    __shared__ __attribute__((aligned(16))) _Float16 mvs[64 * kMvStride];
    __shared__ __attribute__((aligned(16))) _Float16 whi[16 * MT * kWStride], wlo[16 * MT * kWStride];
    __shared__ float Mh[64];
    const LayerGeom &gm = a.geom;
    const int ns = a.n_splits, Hq = a.n_q_heads;
    const int b = blockIdx.y, rg = blockIdx.x;
    const int chunks_total = (seq_blocks(a, b) * gm.G + 63) / 64;  // 64-token chunks of this sequence
    const int chunks_max = (a.n_blocks * gm.G + 63) / 64;          // of the longest one: fixes the ranges
    const int cpr = (chunks_max + a.n_xr - 1) / a.n_xr;
    const int c0 = rg * cpr, c1 = c0 + cpr < chunks_total ? c0 + cpr : chunks_total;
    const int T = seq_blocks(a, b) * gm.G;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, kg = lane >> 4;
    const int ncap = a.tcap / 64 + 1;
    for (int e = tid; e < 16 * MT * kWStride; e += kThreads) whi[e] = wlo[e] = (_Float16)0.0f;
    if (tid < 64) {
        float M = -INFINITY;
        if (tid < Hq)
            for (int sp = 0; sp < ns; sp++)
                M = fmaxf(M, a.ws[(((long long)b * Hq + tid) * ns + sp) * kPartialStride + kHeadDim]);
        Mh[tid] = M;
    }
    __syncthreads();

    // weight staging: thread handles (head tid / 64 + 4 r, token tid % 64) of the chunk
    const int wi = tid >> 6, wt_tok = tid & 63;
    float Mq[NR];
    long long wq[NR];
#pragma unroll
    for (int r = 0; r < NR; r++) {
        const int i = wi + 4 * r < Hq ? wi + 4 * r : 0;
        Mq[r] = Mh[i];
        wq[r] = (long long)b * Hq + i;
    }
    // mean tile staging: thread moves the 16-byte pieces tid + 256 k (row = piece / 16) of the
    // value mean rows of the chunk's tokens; a chunk lies in one or two blocks (or is half of one),
    // whose tiles are looked up once per chunk
    const int G = gm.G, lgG = 31 - __builtin_clz(G); // G is 32, 64 or 128
    const int thr_off = (tid >> 4) * (kHeadDim * 2) + (tid & 15) * 16;
    uint4 mreg[4];
    float xpv[NR], xmv[NR];
    auto fetch = [&](int c) {
#pragma unroll
        for (int r = 0; r < NR; r++) {
            const int t = c * 64 + wt_tok;
            xpv[r] = t < T ? a.xp[wq[r] * a.tcap + t] : 0.0f;
            xmv[r] = a.xmc[wq[r] * ncap + c];
        }
        const int blk0 = (c * 64) >> lgG; // c < chunks_total: the chunk's first block exists
        const unsigned char *tile0 = a.layer + xmean_offset(gm, b, blk0, 1) + (c * 64 - blk0 * G) * (kHeadDim * 2);
        const unsigned char *tile1 = (G < 64 && (blk0 + 1) * G < T) ? a.layer + xmean_offset(gm, b, blk0 + 1, 1) : tile0;
        // piece tid + 256 k is row (tid >> 4) + 16 k: a wave-uniform base per k plus the thread's own offset
#pragma unroll
        for (int k = 0; k < 4; k++) {
            const bool second = 16 * k >= G; // rows 16 k .. 16 k + 15 lie in the chunk's second block
            const unsigned char *base = (second ? tile1 : tile0) + (16 * k - (second ? G : 0)) * (kHeadDim * 2);
            const int t = c * 64 + 16 * k + (tid >> 4);
            mreg[k] = t < T ? *(const uint4 *)(base + thr_off) : uint4{0u, 0u, 0u, 0u};
        }
    };
    v4f acc[MT][2];
#pragma unroll
    for (int mt = 0; mt < MT; mt++) acc[mt][0] = acc[mt][1] = v4f{0.0f, 0.0f, 0.0f, 0.0f};
    if (c0 < c1) fetch(c0);
    for (int c = c0; c < c1; c++) {
        __syncthreads(); // the previous chunk's tiles have been read
#pragma unroll
        for (int r = 0; r < NR; r++) {
            const int i = wi + 4 * r;
            if (i < Hq) {
                const float wt = xpv[r] * exp2f(xmv[r] - Mq[r]);
                const _Float16 hi = (_Float16)wt;
                whi[i * kWStride + wt_tok] = hi;
                wlo[i * kWStride + wt_tok] = (_Float16)(wt - (float)hi);
            }
        }
#pragma unroll
        for (int k = 0; k < 4; k++) {
            const int p = tid + kThreads * k;
            uint2 *dst = (uint2 *)(mvs + (p >> 4) * kMvStride + (p & 15) * 8);
            dst[0] = uint2{mreg[k].x, mreg[k].y};
            dst[1] = uint2{mreg[k].z, mreg[k].w};
        }
        if (c + 1 < c1) fetch(c + 1);
        __syncthreads();
#pragma unroll
        for (int ks = 0; ks < 2; ks++) {
            v8h bm[2];
#pragma unroll
            for (int cc = 0; cc < 2; cc++) {
                const _Float16 *col = mvs + (32 * ks + 8 * kg) * kMvStride + 32 * wave + 16 * cc + n;
#pragma unroll
                for (int j = 0; j < 8; j++) bm[cc][j] = col[j * kMvStride];
            }
#pragma unroll
            for (int mt = 0; mt < MT; mt++) {
                const v8h ahi = *(const v8h *)(whi + (16 * mt + n) * kWStride + 32 * ks + 8 * kg);
                const v8h alo = *(const v8h *)(wlo + (16 * mt + n) * kWStride + 32 * ks + 8 * kg);
#pragma unroll
                for (int cc = 0; cc < 2; cc++) {
                    acc[mt][cc] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ahi, bm[cc], acc[mt][cc], 0, 0, 0);
                    acc[mt][cc] = __builtin_amdgcn_mfma_f32_16x16x32_f16(alo, bm[cc], acc[mt][cc], 0, 0, 0);
                }
            }
        }
    }
    // D: lane holds heads 16 mt + 4 kg .. + 3 of channel 32 wave + 16 cc + n; an empty range stores zeros
#pragma unroll
    for (int mt = 0; mt < MT; mt++)
#pragma unroll
        for (int cc = 0; cc < 2; cc++)
#pragma unroll
            for (int j = 0; j < 4; j++) {
                const int i = 16 * mt + 4 * kg + j;
                if (i < Hq) a.xo[(((long long)b * Hq + i) * a.n_xr + rg) * kHeadDim + 32 * wave + 16 * cc + n] = acc[mt][cc][j];
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

// Workgroups of the value-mean kernel that the device holds at once (0 if the query fails).
template <int MT> static int values_resident()
{
    static const int n = [] {
        int per_cu = 0, dev = 0, cus = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, xhead_values_kernel<MT>, kThreads, 0) != hipSuccess) return 0;
        if (hipGetDevice(&dev) != hipSuccess) return 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
        return per_cu * cus;
    }();
    return n;
}

int xhead_values_resident(int n_q_heads)
{
    const int mt = (n_q_heads + 15) / 16;
    return mt <= 1 ? values_resident<1>() : mt <= 2 ? values_resident<2>() : values_resident<4>();
}

hipError_t launch_xhead_values(const DecodeArgs &a, hipStream_t s)
{
    if (a.n_blocks == 0) return hipSuccess;
    if (a.batch > 65535 || a.n_q_heads > 64 || a.n_xr < 1 || !a.xo) return hipErrorInvalidValue;
    dim3 grid(a.n_xr, a.batch);
    const int mt = (a.n_q_heads + 15) / 16;
    (void)hipGetLastError(); // drop any stale error left by earlier runtime calls of this thread
    if (mt <= 1) hipLaunchKernelGGL(xhead_values_kernel<1>, grid, dim3(kThreads), 0, s, a);
    else if (mt <= 2) hipLaunchKernelGGL(xhead_values_kernel<2>, grid, dim3(kThreads), 0, s, a);
    else hipLaunchKernelGGL(xhead_values_kernel<4>, grid, dim3(kThreads), 0, s, a);
    return note_launch(hipGetLastError());
}

} // namespace tadakv
