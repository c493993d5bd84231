// Decode attention over the packed cache on the matrix cores (gfx950, v_mfma_i32_16x16x64_i8).
//
// What is computed is the same as in the vector-ALU kernel (arxiv 2506.04642 Eq. 5-8, flash
// decoding of App. A): per block
//   score_t = ( sum_c (q_c s_c) code_tc + sum_c q_c (z_c + m_c) ) / sqrt(d)
//   o_c     = sum_t (p_t s_tg) code_tc + sum_t p_t z_tg + m_c sum_t p_t
// but the two contractions over codes run as int8 matrix products.  The small operand
// (q_c s_c per block, p_t s_tg per 64-token chunk) is converted to 23-bit fixed point against a
// power-of-two bound and split into three signed bytes ("limbs"); the 16 rows of the matrix
// instruction hold (query head, limb) for four query heads, and a kv head with more than four
// query heads is served as two such head groups that share the unpacked codes.  The codes are
// the other operand: one shift and one mask turn a 32-bit word of the cache into four int8
// codes, which is why the storage format interleaves fields bytewise.  Products and sums are
// exact in int32; the only rounding is the fixed-point conversion (relative 2^-23 of the chunk's
// largest weight).
//
// Work split: one workgroup (NW waves) per (sequence, kv head, split).  Each wave owns every
// NW-th 64-token chunk of the split and keeps its own online-softmax state; the states are
// merged through LDS at the end and one partial (max, sum, output) per query head is written for
// the cross-split merge kernel.  Waves never synchronise inside the main loop: every LDS buffer
// in the loop is private to a wave.
//
// Memory pipeline: the records of a chunk are contiguous in the cache, so a chunk is fetched as
// one linear run of 16-byte pieces straight into the wave's LDS staging buffer
// (global_load_lds_dwordx4, no vector registers involved).  A wave copies the staged chunk into
// registers, immediately issues the fetch of its next chunk into the same buffer, and only then
// computes, so the HBM latency of chunk i+1 is covered by the arithmetic of chunk i.
//
// Lane roles inside a wave (lane = 16*row + n, quad position qa = n & 3, quad index vq = n >> 2):
//   matrix output      lane (row, n): query head 4*hg + row, limbs in the four accumulator
//                      registers; column n = token n of a 16-token tile (keys) or channel n of a
//                      16-channel tile (values).
//   key-side producer  lane (row, vq, qa): head 4*hg + row, channels 32*vq + 16*ph + 4*qa + {0..3}.
//   matrix operands    lane (row, n): operand row / column n, 16 consecutive k-slots of group `row`.
#include "tadakv_internal.h"
#include <hip/hip_ext.h>
#include <hip/hip_fp16.h>

namespace tadakv {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int kWavesPerBlock = 4;
constexpr float kScoreScale = 0.08838834764831845f * 1.4426950408889634f; // log2(e) / sqrt(128)
constexpr uint32_t kM4 = 0x0F0F0F0Fu, kM2 = 0x03030303u;

template <int CTRL> __device__ __forceinline__ uint32_t dpp_u(uint32_t x)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, 0xF, 0xF, true);
}
template <int CTRL> __device__ __forceinline__ float dpp_f(float x)
{
    return __uint_as_float(dpp_u<CTRL>(__float_as_uint(x)));
}
// quad_perm [1,0,3,2] = 0xB1, [2,3,0,1] = 0x4E, row_half_mirror = 0x141, row_mirror = 0x140:
// after the four steps every lane of a row of 16 holds the row's total
__device__ __forceinline__ float row_sum(float x)
{
    x += dpp_f<0xB1>(x);
    x += dpp_f<0x4E>(x);
    x += dpp_f<0x141>(x);
    x += dpp_f<0x140>(x);
    return x;
}
__device__ __forceinline__ float row_max(float x)
{
    x = fmaxf(x, dpp_f<0xB1>(x));
    x = fmaxf(x, dpp_f<0x4E>(x));
    x = fmaxf(x, dpp_f<0x141>(x));
    x = fmaxf(x, dpp_f<0x140>(x));
    return x;
}
__device__ __forceinline__ uint32_t pk_max_u16(uint32_t a, uint32_t b)
{
    typedef unsigned short us2 __attribute__((ext_vector_type(2)));
    const us2 x = __builtin_bit_cast(us2, a), y = __builtin_bit_cast(us2, b);
    const us2 m = __builtin_elementwise_max(x, y);
    return __builtin_bit_cast(uint32_t, m);
}
__device__ __forceinline__ uint32_t row_pk_max_u16(uint32_t x)
{
    x = pk_max_u16(x, dpp_u<0xB1>(x));
    x = pk_max_u16(x, dpp_u<0x4E>(x));
    x = pk_max_u16(x, dpp_u<0x141>(x));
    x = pk_max_u16(x, dpp_u<0x140>(x));
    return x;
}

__device__ __forceinline__ float widen16(uint16_t v, int dtype)
{
    if (dtype == 1) return __uint_as_float((uint32_t)v << 16);
    return __half2float(__ushort_as_half(v));
}
__device__ __forceinline__ float h_lo(uint32_t w) { return __half2float(__ushort_as_half((uint16_t)(w & 0xFFFFu))); }
__device__ __forceinline__ float h_hi(uint32_t w) { return __half2float(__ushort_as_half((uint16_t)(w >> 16))); }
__device__ __forceinline__ half2_t as_h2(uint32_t w) { return __builtin_bit_cast(half2_t, w); }

// power of two strictly above x (x >= 0) but at least 2 * floor_v
__device__ __forceinline__ float pow2_above(float x, float floor_v)
{
    return __uint_as_float((__float_as_uint(fmaxf(x, floor_v)) & 0x7F800000u) + 0x00800000u);
}

// waits for this wave's outstanding LDS traffic and keeps the compiler from moving LDS accesses
// across; enough to hand data between lanes of one wave through LDS
__device__ __forceinline__ void wave_lds_fence() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

__device__ __forceinline__ v4i mfma(v4i a, v4i b, v4i c)
{
    return __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, c, 0, 0, 0);
}
// three signed-byte limbs (weights 1, 256, 65536) -> float.  The two upper limbs are combined in
// integer (no overflow: a limb sum is below 2^23), so the conversion rounds once, at 2^-24 relative.
__device__ __forceinline__ float limbs_to_float(v4i acc)
{
    return (float)acc.x + 256.0f * (float)(acc.y + (acc.z << 8));
}
// Hides a value's origin from the optimiser: without this a constant of the form (C - m) that is
// added to many values is re-associated into two operations per value.
__device__ __forceinline__ uint32_t opaque(uint32_t x)
{
    asm volatile("" : "+v"(x));
    return x;
}
// power of two strictly above the larger of the two non-negative binary16 values in w (at least
// 2^-14), straight from the exponent field
__device__ __forceinline__ float pow2_above_h2(uint32_t w, bool both)
{
    const uint32_t m = both ? max(w & 0xFFFFu, w >> 16) : (w & 0xFFFFu);
    return __uint_as_float(((m & 0x7C00u) << 13) + (113u << 23)); // value exponent (e5 - 15) + 1, biased by 127
}

// running softmax state of one lane for one query head; O for channels 16*ct + n
struct State {
    float M, l;      // running max (exp2 domain), lane-partial sum of weights
    float O[8];      // output accumulators
    float Zp[4];     // lane-partial sum_t p_t z_{t,gamma}
};

// Online-softmax bookkeeping for one chunk of up to 64 tokens: s[k] is the score (exp2 domain)
// of token 16k + n or -inf.  Returns p[k] relative to the chunk's own max, and the factors
// alpha (old state) and wc (this chunk) that bring both to the new running max.
__device__ __forceinline__ void softmax_chunk(const float (&s)[4], State &st, float (&p)[4], float &alpha,
                                              float &wc, float &mc)
{
    mc = fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3]));
    mc = row_max(mc);
    const float m_new = fmaxf(st.M, mc);
    // the bare instruction: arguments are <= 0 (or -inf), and a weight below 2^-126 may flush to zero
    alpha = __builtin_amdgcn_exp2f(st.M - m_new);
    wc = __builtin_amdgcn_exp2f(mc - m_new);
    st.M = m_new;
#pragma unroll
    for (int k = 0; k < 4; k++) p[k] = __builtin_amdgcn_exp2f(s[k] - mc);
    st.l = st.l * alpha + wc * ((p[0] + p[1]) + (p[2] + p[3]));
}

// Record layout for one template instance; must agree with the layer geometry built on the host.
// B: the code width; layers whose keys and values differ in width carry both, keys' | values' << 4
// (kbits_of, vbits_of)
constexpr int kbits_of(int B) { return B & 15; }
constexpr int vbits_of(int B) { return (B >> 4) ? (B >> 4) : (B & 15); }
template <int B, int G, int GC, bool MEAN> struct RecLayout {
    static constexpr int KC = G * kHeadDim * kbits_of(B) / 8; // bytes of key codes
    static constexpr int VC = G * kHeadDim * vbits_of(B) / 8; // bytes of value codes
    static constexpr int K_CODES = 0;
    static constexpr int K_SCALE = KC;
    static constexpr int K_ZERO = KC + 256;
    static constexpr int K_MEAN = KC + 512;
    static constexpr int V_CODES = KC + 512 + (MEAN ? 256 : 0);
    static constexpr int V_META = V_CODES + VC;
    static constexpr int V_MEAN = V_META + G * (kHeadDim / GC) * 4;
    static constexpr int REC = (V_MEAN + (MEAN ? 256 : 0) + 255) / 256 * 256;
    static bool matches(const LayerGeom &g)
    {
        return g.rec_bytes == REC && g.k_codes == K_CODES && g.k_scale == K_SCALE && g.k_zero == K_ZERO &&
               (!MEAN || g.k_mean == K_MEAN) && g.v_codes == V_CODES && g.v_meta == V_META &&
               (!MEAN || g.v_mean == V_MEAN);
    }
};

// Fetch NBYTES (multiple of 16) from src to the LDS address dst; both wave-uniform.  Lane l moves
// the 16-byte pieces l, l + 64, ...; completion is tracked by the vector-memory counter.
// The fetches are issued by hand (direct-to-LDS loads: lane l's 16 bytes land at M0 + offset + 16 l,
// the offset applies to the global and to the LDS address alike).  The compiler does not see them:
// through the builtin it makes every LDS access that it cannot tell apart from a fetch's destination
// wait for ALL outstanding fetches, the wave's next chunk included, which is exactly the overlap
// this kernel lives on.  Every read of a staged buffer therefore follows a wait written here
// (stage_wait, stage_wait_but).
template <int OFF> __device__ __forceinline__ void stage_fetch16(const unsigned char *gp, uint32_t lds)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off offset:%2"
                 : : "s"(lds), "v"(gp), "n"(OFF) : "memory", "m0");
}
template <int NBYTES>
__device__ __forceinline__ void stage_issue(const unsigned char *src, uint32_t *dst, int lane)
{
#pragma unroll
    for (int base = 0; base < NBYTES; base += 4096) {
        const unsigned char *gp = src + base + lane * 16;
        const uint32_t lp = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(uintptr_t)(__attribute__((address_space(3))) void *)(dst + base / 4));
        if (base + 0 * 1024 + 1024 <= NBYTES) stage_fetch16<0>(gp, lp);
        else if (base + 0 * 1024 < NBYTES && base + lane * 16 < NBYTES) stage_fetch16<0>(gp, lp);
        if (base + 1 * 1024 + 1024 <= NBYTES) stage_fetch16<1024>(gp, lp);
        else if (base + 1 * 1024 < NBYTES && base + 1024 + lane * 16 < NBYTES) stage_fetch16<1024>(gp, lp);
        if (base + 2 * 1024 + 1024 <= NBYTES) stage_fetch16<2048>(gp, lp);
        else if (base + 2 * 1024 < NBYTES && base + 2048 + lane * 16 < NBYTES) stage_fetch16<2048>(gp, lp);
        if (base + 3 * 1024 + 1024 <= NBYTES) stage_fetch16<3072>(gp, lp);
        else if (base + 3 * 1024 < NBYTES && base + 3072 + lane * 16 < NBYTES) stage_fetch16<3072>(gp, lp);
    }
}
__device__ __forceinline__ void stage_wait() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
// dense binary16 product on the matrix cores (v_mfma_f32_16x16x32_f16), operands as 16 raw bytes
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ v4f mfma_h(const u32x4 &a, const u32x4 &b, v4f c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(v8h, a), __builtin_bit_cast(v8h, b), c, 0, 0, 0);
}
// LDS reads issued by hand, for data read while a direct-to-LDS fetch is outstanding: the compiler
// makes an LDS read that it cannot tell apart from the fetch's destination wait for ALL of the wave's
// outstanding fetches (its next chunk included).  A result must not be used before lds_wait and then
// lds_got of the register.
template <int OFF> __device__ __forceinline__ void lds_get16(u32x4 &dst, uint32_t addr)
{
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(OFF));
}
__device__ __forceinline__ void lds_wait() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }
__device__ __forceinline__ void lds_got(u32x4 &r) { asm volatile("" : "+v"(r)); }
__device__ __forceinline__ uint32_t lds_addr(const void *p)
{
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void *)p;
}
// Progress counters in LDS, one per wave of a workgroup, for exchanges that are not fenced by a
// barrier: a wave publishes how far it has come (after its own LDS traffic has completed), and a
// wave that needs the others' data polls until every counter has reached what it needs.  All waves
// of a workgroup are resident together and the wave that is furthest behind never waits (it needs
// nothing that a wave ahead of it has yet to produce), so every wait ends; the spin limit is a
// second line of defence only.
__device__ __forceinline__ void progress_publish(uint32_t addr, uint32_t val, int lane)
{
    wave_lds_fence();
    if (lane == 0) asm volatile("ds_write_b32 %0, %1" : : "v"(addr), "v"(val) : "memory");
}
template <int NW> __device__ __forceinline__ void progress_wait_all(uint32_t base, uint32_t need, int lane)
{
    const uint32_t ea = base + 4 * (lane & (NW - 1));
    for (int spin = 0; spin < (1 << 20); spin++) {
        uint32_t v;
        asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(ea) : "memory");
        if (__builtin_amdgcn_ballot_w64(v < need) == 0) break;
        __builtin_amdgcn_s_sleep(1);
    }
}
// Global loads issued by hand, for data wanted long after younger fetches have been issued under a
// condition: the compiler, which has to assume either outcome of the condition, would wait for
// every outstanding fetch before the first use.  A result must not be used before glb_wait_but
// (N = the number of fetches issued since, which may stay outstanding) and then glb_got of every
// register.
// Between the request and the hand-over the compiler takes the destination for a value that exists:
// under register pressure it may move it (into another register, into the accumulation file), and
// then the data arrives in a register that has been given to something else -- an address, say.
// The destinations are therefore accumulation registers, of which these kernels use few: nothing
// competes for them, they take no part in the pressure on the ordinary file, and what needs the data
// in an ordinary register copies it after the hand-over.  The build reads the generated code and
// refuses it if any instruction between a request and its hand-over names a destination.
__device__ __forceinline__ void glb_get16(u32x4 &dst, const void *p)
{
    asm volatile("global_load_dwordx4 %0, %1, off ; by hand" : "=a"(dst) : "v"(p));
}
// (the wait and the hand-over of the registers are separate so that a wait chosen by a condition
// is followed by ONE hand-over per register: registers handed over on either side of a branch would
// be copied into common ones ahead of the branch, that is, before the data is there)
template <int N> __device__ __forceinline__ void glb_wait_but()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a six-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}
__device__ __forceinline__ void glb_got(u32x4 &r) { asm volatile("; by hand %0" : "+a"(r) : : "memory"); }
// Blocks of 128 tokens are read as two halves of 64: the pieces of half hf of the record at src
// (its key codes, the block's key metadata, its runs of value codes -- 1 KiB per group of channel
// tiles --, its value metadata, the block's value mean) are placed so that the staging buffer
// holds the image of a 64-token record, which is what the arithmetic below works on.  A wave
// takes the two halves of a block one after the other; the pieces they share are fetched with the
// first (shared) and stay in the buffer for the second.
template <int B, int GC, bool MEAN>
__device__ __forceinline__ void stage_issue_half(const unsigned char *src, int hf, bool shared, uint32_t *dst, int lane)
{
    typedef RecLayout<B, 64, GC, MEAN> RL;   // the image
    typedef RecLayout<B, 128, GC, MEAN> RS;  // the record
    constexpr int NG = kHeadDim / GC;
    static_assert(RS::KC == 2 * RL::KC && RL::KC % 1024 == 0 && RL::KC == RL::VC, "code halves (one width for keys and values)");
    stage_issue<RL::KC>(src + RS::K_CODES + hf * RL::KC, dst + RL::K_CODES / 4, lane);
    if (shared) stage_issue<512 + (MEAN ? 256 : 0)>(src + RS::K_SCALE, dst + RL::K_SCALE / 4, lane);
#pragma unroll
    for (int r = 0; r < RL::KC / 1024; r++)
        stage_issue<1024>(src + RS::V_CODES + (2 * r + hf) * 1024, dst + (RL::V_CODES + r * 1024) / 4, lane);
    stage_issue<64 * NG * 4>(src + RS::V_META + hf * 64 * NG * 4, dst + RL::V_META / 4, lane);
    if (MEAN && shared) stage_issue<256>(src + RS::V_MEAN, dst + RL::V_MEAN / 4, lane);
}

// int8 operand of the matrix instruction for the codes held in a lane
template <int B> struct CodeOps;
template <> struct CodeOps<4> { // two words = one tile line of 16 codes
    static __device__ __forceinline__ v4i line(uint32_t w0, uint32_t w1)
    {
        return v4i{(int)(w0 & kM4), (int)((w0 >> 4) & kM4), (int)(w1 & kM4), (int)((w1 >> 4) & kM4)};
    }
};
// Phase clocks (a build with -DTADA_PHASE_CLOCK only; the library proper carries none of it): every
// wave sums the cycles between the marks of the main loop; kv_debug_phase_clocks hands the sums out.
#ifdef TADA_PHASE_CLOCK
__device__ unsigned long long tada_phase_clk[16];
#define PHASE_INIT unsigned long long pclk_[14] = {}; unsigned long long plast_ = __builtin_readcyclecounter(); int piter_ = 0;
#define PHASE(i) { const unsigned long long t_ = __builtin_readcyclecounter(); pclk_[i] += t_ - plast_; plast_ = t_; }
#define PHASE_ITER piter_++;
#define PHASE_DONE if (lane == 0) { for (int i_ = 0; i_ < 14; i_++) atomicAdd(&tada_phase_clk[i_], pclk_[i_]); \
                                    atomicAdd(&tada_phase_clk[14], (unsigned long long)piter_); atomicAdd(&tada_phase_clk[15], 1ull); }
#else
#define PHASE_INIT
#define PHASE(i)
#define PHASE_ITER
#define PHASE_DONE
#endif

template <> struct CodeOps<2> { // one word = one tile line
    static __device__ __forceinline__ v4i line(uint32_t w)
    {
        return v4i{(int)(w & kM2), (int)((w >> 2) & kM2), (int)((w >> 4) & kM2), (int)((w >> 6) & kM2)};
    }
};
template <> struct CodeOps<8> { // four words = one tile line; split into nibbles to stay inside int8
    static __device__ __forceinline__ v4i lo(uint4 w)
    {
        return v4i{(int)(w.x & kM4), (int)(w.y & kM4), (int)(w.z & kM4), (int)(w.w & kM4)};
    }
    static __device__ __forceinline__ v4i hi(uint4 w)
    {
        return v4i{(int)((w.x >> 4) & kM4), (int)((w.y >> 4) & kM4), (int)((w.z >> 4) & kM4), (int)((w.w >> 4) & kM4)};
    }
};

// XH: cross-head mean.  The records carry no mean (MEAN is false).
//   XH == 1: the mean's share of every score comes in through a.xs, and the softmax weights go out
//            through a.xp / a.xmc for the kernel that adds the value mean plane's share to the
//            partial outputs (two more kernels and a round trip of scores and weights).
//   XH == 2: both mean terms inside this kernel.  A workgroup is one (sequence, split) and NW kv
//            heads (all of them, or half: then two workgroups share the split), a wave per kv head:
//            every wave takes the same chunks, each of its own head's records.  The mean rows of a
//            chunk (64 tokens x 128 channels of binary16 for keys and for values, shared by all kv
//            heads: Eq. 1-2) go from global memory straight into matrix-core operands: q . mean_K and
//            sum_t p_t mean_V[t] are dense binary16 products (queries narrowed to binary16: exact in
//            its normal range; weights as a binary16 pair hi + lo; binary32 accumulation) that the
//            waves share out among themselves -- the scores by (16 query heads, 16 tokens), the
//            value share by 16-channel tile for all heads -- and whose small operands and results
//            (scores, weights, rescale factors) they exchange through LDS, paced by per-wave
//            progress counters instead of barriers.
// PG: paged placement (block slots through a table); the dense instances carry none of its state.
// GS: tokens per block of the cache (32, 64, or 128 read as two halves of 64).
template <int B, int GS, int GC, bool MEAN, int NW, int NHG, int XH, bool PG>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu((B == 2 && NHG == 1 && !XH) ? (PG ? 3 : 4) : 1, 8))) void decode_split_mfma_kernel(DecodeArgs a)
{
    static_assert(!(XH && MEAN), "cross-head layers store no per-record mean");
    constexpr bool XF = XH == 2; // both mean terms in this kernel, a wave per kv head
    constexpr int CW = XF ? 1 : NW;          // waves that share a unit's chunks
    constexpr int XSL = 3;                   // copies of every exchange buffer of the fused cross-head form
    constexpr bool H2 = GS == 128;         // a block is worked on as two halves
    constexpr int G = H2 ? 64 : GS;        // tokens per block as the arithmetic sees it
    constexpr int HB = GS / G;             // such blocks per block of the cache
    typedef RecLayout<B, G, GC, MEAN> RL;  // the staged image
    constexpr int SREC = RecLayout<B, GS, GC, MEAN>::REC; // bytes of a record in the cache
    constexpr int NBC = 64 / G;            // blocks per 64-token chunk
    constexpr int TPB = G / 16;            // 16-token tiles per block
    constexpr int NG = kHeadDim / GC;      // value scale groups
    constexpr int TPG = GC / 16;           // channel tiles per value scale group
    constexpr int KB = kbits_of(B), VB = vbits_of(B);       // code widths of keys and of values
    constexpr int NKL = (KB == 4) ? 4 : (KB == 2 ? 2 : 8); // key code pieces per lane and chunk
    constexpr int NVL = (VB == 4) ? 4 : (VB == 2 ? 2 : 8); // value code pieces per lane and chunk
    constexpr int REC = RL::REC;
    constexpr int CB = NBC * REC;          // bytes of one chunk
    constexpr int STAGE_DW = CB / 4;       // staging buffer of a wave
    // operand scratch, reused block after block and pass after pass: key operands of one block
    // [NHG][2 phases][64 lanes][4], value operands of NGP scale groups [NHG][NGP][64 lanes][4]
    constexpr int NGP = NG > 2 ? 2 : NG;
    constexpr int AK_DW = NHG * 512, AV_DW = NHG * NGP * 256;
    constexpr int OPER_DW = AK_DW > AV_DW ? AK_DW : AV_DW;
    constexpr int WAVE_DW = STAGE_DW + OPER_DW;
    // fused cross-head form: the workgroup's query heads, 4 NHG per kv head (wave), as 16-head blocks
    constexpr int HP = 4 * NHG, HQP = NW * HP, NRB = XF ? HQP / 16 : 1;
    constexpr int NCT = XF ? 8 / NW : 1;    // channel tiles of the value-mean product per wave
    constexpr int PB_ROW = 144;             // bytes of a row of 64 binary16 (+ 8 of padding)
    // shared by the waves, all [chunk mod 3]...: scores q . mean_K [head][64 tokens] binary32 (the
    // 16-token groups of a row rotated by the head so that writers and readers spread over the banks),
    // softmax weights [hi | lo][head][64 + 8] binary16, rescale factors [head]; and a progress counter
    // per wave (the chunks it has finished)
    constexpr int XS_DW = XF ? XSL * HQP * 64 : 0, PB_DW = XF ? XSL * 2 * HQP * PB_ROW / 4 : 0, AL_DW = XF ? XSL * HQP : 0;
    constexpr int LDS_DW = NW * WAVE_DW;

    __shared__ __attribute__((aligned(16))) uint32_t lds_all[LDS_DW];
    // the exchange buffers of the fused cross-head form
    __shared__ __attribute__((aligned(16))) uint32_t lds_xs[XF ? XS_DW : 1], lds_pb[XF ? PB_DW : 1], lds_al[XF ? AL_DW : 1],
        lds_ev[XF ? 16 : 1];

    const LayerGeom &gm = a.geom;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6); // wave-uniform: lets addresses live in scalars
    const int row = lane >> 4, n = lane & 15, qa = lane & 3, vq = (lane >> 2) & 3;
    uint32_t *lds = lds_all + wave * WAVE_DW;
    uint32_t *stage = lds;                 // the chunk as it lies in the cache
    uint32_t *ak = lds + STAGE_DW, *av = ak;

    // fused cross-head form: a workgroup takes NW kv heads of a sequence; with more heads several
    // workgroups (parts) share a (sequence, split) and read the same mean rows -- they sit 8 apart in
    // the launch order when the split count allows (same XCD and so the same L2, resident together)
    const int parts = XF ? a.n_kv_heads / NW : 1;
    int sp = blockIdx.x, half = 0; // half: which part
    if (XF && parts > 1) {
        if (a.n_splits % 8 == 0) {
            half = (sp >> 3) % parts;
            sp = (sp & 7) | (((sp >> 3) / parts) << 3);
        } else {
            half = sp % parts;
            sp /= parts;
        }
    }
    const int u = XF ? (int)blockIdx.y * a.n_kv_heads + half * NW + wave : (int)blockIdx.y;
    const int b = u / a.n_kv_heads, h = u % a.n_kv_heads;
    const int g = a.g;
    const int cw0 = XF ? 0 : wave; // this wave's first local chunk

    // rows 4i+3 of the operands (the unused fourth limb) must read as zero
    for (int i = lane; i < OPER_DW; i += 64) ak[i] = 0u;

    // ---- chunks of this split: the splits of a unit interleave chunk by chunk (split sp, wave w
    // takes chunks sp + n_splits * (w + NW * k)), so that together they sweep the unit's records
    // front to back as one moving window instead of as n_splits far-apart streams
    const int b_end = seq_blocks(a, b) * HB, r_seq = seq_resid(a, b); // this sequence's packed blocks and raw tokens
    const int chunks_total = (b_end + NBC - 1) / NBC;
    const int ns = a.n_splits;
    // local chunk j of this split is the unit's chunk sp + ns * j
    const int w0 = sp * NBC;          // first block of local chunk 0
    const int cstride = ns * NBC;     // blocks between consecutive local chunks
    // H2: the splits interleave block by block, and a wave's chunks 2 k and 2 k + 1 are the two
    // halves of its k-th block; n_chunks is then the wave's own bound (cw0 + CW * its chunks; the
    // CW waves that share a unit's chunks: all of the workgroup's, or, in the fused cross-head form,
    // this one alone)
    const int blocks_sp = sp * HB < chunks_total ? (chunks_total / HB - sp + ns - 1) / ns : 0; // H2 only
    const int n_chunks = H2 ? cw0 + CW * 2 * ((blocks_sp - cw0 + CW - 1) / CW)
                            : (sp < chunks_total ? (chunks_total - sp + ns - 1) / ns : 0);
    // first block (as the arithmetic counts them) of this wave's local chunk ci = cw0 + CW * k
    auto blk_of = [&](int ci) {
        if (!H2) return w0 + ci * cstride;
        const int k = (ci - cw0) / CW;
        return 2 * (sp + ns * (cw0 + CW * (k >> 1))) + (k & 1);
    };
    const unsigned char *unit_base = a.layer + (long long)u * gm.NB * SREC;

    // Paged placement: lane l keeps the slots of the blocks of this wave's chunk number slot_base + l
    // (one table read per 64 chunks of the wave), so that the fetch of a chunk waits for no lookup.
    int slotv[NBC], slot_base = 0;
    auto load_slots = [&](int it0) {
        slot_base = it0;
        const int blk0 = blk_of(cw0 + CW * (it0 + lane));
#pragma unroll
        for (int bi = 0; bi < NBC; bi++) {
            int blk = blk0 + bi < b_end ? blk0 + bi : blk0; // no second block: the first one again
            blk = blk < b_end ? blk : b_end - 1;            // chunks past the end: any block the sequence has
            slotv[bi] = blk >= 0 ? (int)block_slot(gm, b, blk / HB) : 0;
        }
    };
    if (PG) load_slots(0);

    auto issue = [&](int ci) {
        const int blk0 = blk_of(ci);
        if (PG) {
            // every block of the chunk has a place of its own
            const int it = (ci - cw0) / CW;
            if (it - slot_base >= 64) load_slots(it); // (the fused cross-head form moves the window itself)
#pragma unroll
            for (int bi = 0; bi < NBC; bi++) {
                const long long slot = __builtin_amdgcn_readlane(slotv[bi], it - slot_base);
                const unsigned char *rec = a.layer + (slot * a.n_kv_heads + h) * SREC;
                if constexpr (H2) stage_issue_half<B, GC, MEAN>(rec, blk0 & 1, !(blk0 & 1), stage, lane);
                else stage_issue<REC>(rec, stage + bi * (REC / 4), lane);
            }
            return;
        }
        const unsigned char *src = unit_base + (long long)(blk0 / HB) * SREC;
        if constexpr (H2) {
            stage_issue_half<B, GC, MEAN>(src, blk0 & 1, !(blk0 & 1), stage, lane);
        } else if (NBC == 1 || blk0 + 1 < b_end) {
            stage_issue<CB>(src, stage, lane);
        } else {
            // the chunk's second block does not exist: stage the first one twice so that the
            // (masked) arithmetic on the second half still sees finite numbers
            stage_issue<REC>(src, stage, lane);
            stage_issue<REC>(src, stage + (NBC - 1) * (REC / 4), lane);
        }
    };
    // the query words are requested ahead of the first chunk: loads return in order, and the
    // query is worked on while the chunk is still on its way
    uint2 qraw[NHG][2];
#pragma unroll
    for (int hg = 0; hg < NHG; hg++) {
        const int head = 4 * hg + row;
        const uint16_t *qp = a.q + ((long long)b * a.n_q_heads + h * g + (head < g ? head : 0)) * kHeadDim;
#pragma unroll
        for (int ph = 0; ph < 2; ph++) qraw[hg][ph] = *(const uint2 *)(qp + 32 * vq + 16 * ph + 4 * qa);
    }
    if (cw0 < n_chunks) issue(cw0);
    // fused cross-head form: row r (token of the chunk that starts with block blk0) of the key (which
    // = 0) or value (1) mean plane.  The second block of a chunk that does not exist is read as the first.
    // (it: the number of that chunk among this wave's, for the slots under paged placement)
    auto mean_row_src = [&](int which, int blk0, int r, int it) {
        int blk = blk0 + r / G;
        blk = blk < b_end ? blk : blk0;
        // block slot = sequence * blocks per sequence + block, or what the table says; with blocks of
        // 128 tokens blk counts their halves
        long long slot;
        if (PG) {
            const int s0 = __builtin_amdgcn_readlane(slotv[0], it - slot_base);
            const int s1 = __builtin_amdgcn_readlane(slotv[NBC - 1], it - slot_base);
            slot = r / G == 0 ? s0 : s1;
        } else {
            slot = (long long)b * gm.NB + blk / HB;
        }
        return a.layer + gm.xmean_off + ((slot * 2 + which) * GS + (blk % HB) * G + r % G) * (kHeadDim * 2);
    };

    // ---- query of heads 4*hg + row: this lane's eight channels, widened and as binary16 pairs
    float qf[NHG][2][4];      // q, widened (exact)
    half2_t qh[NHG][2][2];    // the same as binary16 pairs for the zero / mean dot products
    float three_qb[NHG];      // 3 qb, qb = power of two above max |q| of the head
    float inv_kf_base[NHG];   // qb 2^-22 log2(e)/sqrt(d): one fixed-point step, up to the scale bound
#pragma unroll
    for (int hg = 0; hg < NHG; hg++) {
        const int head = 4 * hg + row;
        float qmax = 0.0f;
#pragma unroll
        for (int ph = 0; ph < 2; ph++)
#pragma unroll
            for (int y = 0; y < 4; y++) {
                const uint32_t w = (y & 2) ? qraw[hg][ph].y : qraw[hg][ph].x;
                const uint16_t q16 = (uint16_t)((y & 1) ? (w >> 16) : (w & 0xFFFFu));
                qf[hg][ph][y] = head < g ? widen16(q16, gm.dtype) : 0.0f;
                qmax = fmaxf(qmax, fabsf(qf[hg][ph][y]));
            }
        qmax = row_max(qmax);
        const float qb = pow2_above(qmax, 0x1p-60f);
        three_qb[hg] = 3.0f * qb;
        inv_kf_base[hg] = qb * 0x1p-22f * kScoreScale;
#pragma unroll
        for (int ph = 0; ph < 2; ph++) {
            qh[hg][ph][0] = half2_t{(_Float16)qf[hg][ph][0], (_Float16)qf[hg][ph][1]};
            qh[hg][ph][1] = half2_t{(_Float16)qf[hg][ph][2], (_Float16)qf[hg][ph][3]};
        }
    }

    State st[NHG];
#pragma unroll
    for (int hg = 0; hg < NHG; hg++) {
        st[hg].M = -INFINITY;
        st[hg].l = 0.0f;
#pragma unroll
        for (int k = 0; k < 8; k++) st[hg].O[k] = 0.0f;
#pragma unroll
        for (int k = 0; k < 4; k++) st[hg].Zp[k] = 0.0f;
    }
    wave_lds_fence();

    // ---- fused cross-head form.  The mean terms are dense products that the whole workgroup shares:
    // q . mean_K for all its query heads, 16 heads x 16 tokens per matrix product, dealt to the waves by
    // (head block, token tile) -- wave w takes the pairs w NHG + e --, and sum_t p_t mean_V[t] by
    // channel tile, every wave for all heads.  The waves exchange the small operands and results
    // (scores, weights, rescale factors) through LDS without a barrier: a wave publishes the number
    // of chunks it has finished and waits, once per chunk, until every wave has finished the previous
    // one.  The scores of chunk i + 2 are worked out at the end of chunk i, the value-mean product of
    // chunk i - 1 runs at the end of chunk i, and every exchange buffer exists three times (chunk mod
    // 3): no wave gets more than one chunk ahead of another, and none overwrites what another still
    // reads.  (With a barrier per chunk a wave that waits for the slowest chunk of the round leaves
    // its SIMD idle: 329 against 262 us per 8-bit layer on 16 sequences of 32768 tokens.)
    u32x4 qA[NHG][4];  // A operands of the score products: row = head of the block, binary16
    int xs_w[NHG], xs_t0[NHG], xs_r[NHG], xs_rot[NHG]; // where this lane's scores are written and read (float index)
    int km_row[NHG];   // this lane's row (token of the chunk) of the key-mean tile as B operand
    v4f accv[NRB][NCT]; // sum_t p_t mean_V[t] (times 2^8) of heads 16 rb + 4 row + j, channel 16 (w NCT + c) + n
    auto kmean_fetch = [&](u32x4 (&kb)[NHG][4], int blk0, int it) {
#pragma unroll
        for (int e = 0; e < NHG; e++)
#pragma unroll
            for (int ks = 0; ks < 4; ks++) glb_get16(kb[e][ks], mean_row_src(0, blk0, km_row[e], it) + 64 * ks + 16 * row);
    };
    auto kmean_scores = [&](const u32x4 (&kb)[NHG][4], int sl) {
        float *xs = (float *)lds_xs + sl * (HQP * 64);
#pragma unroll
        for (int e = 0; e < NHG; e++) {
            v4f acc = v4f{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int ks = 0; ks < 4; ks++) acc = mfma_h(qA[e][ks], kb[e][ks], acc);
#pragma unroll
            for (int j = 0; j < 4; j++) xs[xs_w[e] + j * 64 + (((xs_t0[e] + j) & 3) << 4)] = acc[j];
        }
    };
    if (XF) {
#pragma unroll
        for (int e = 0; e < NHG; e++) {
            const int pj = wave * NHG + e, rb = pj >> 2, tt = pj & 3; // head block, token tile
            const int hp = 16 * rb + n, hk = half * NW + hp / HP, local = hp % HP; // A row n: kv head, head of its group
            const uint16_t *qp = a.q + ((long long)b * a.n_q_heads + hk * g + (local < g ? local : 0)) * kHeadDim + 8 * row;
#pragma unroll
            for (int ks = 0; ks < 4; ks++) {
                const uint4 w = *(const uint4 *)(qp + 32 * ks);
                const uint32_t wv[4] = {w.x, w.y, w.z, w.w};
                uint32_t o[4];
#pragma unroll
                for (int k = 0; k < 4; k++) {
                    const _Float16 lo = (_Float16)widen16((uint16_t)(wv[k] & 0xFFFFu), gm.dtype);
                    const _Float16 hi = (_Float16)widen16((uint16_t)(wv[k] >> 16), gm.dtype);
                    o[k] = local < g ? (uint32_t)__builtin_bit_cast(uint16_t, lo) | ((uint32_t)__builtin_bit_cast(uint16_t, hi) << 16) : 0u;
                }
                qA[e][ks] = u32x4{o[0], o[1], o[2], o[3]};
            }
            km_row[e] = 16 * tt + n;
            // result register j: head 16 rb + 4 row + j, token 16 tt + n; the 16-token groups of head
            // hp's row are rotated by (hp % 4 + hp / 4) % 4
            xs_w[e] = (16 * rb + 4 * row) * 64 + n;
            xs_t0[e] = (tt + row) & 3;
        }
#pragma unroll
        for (int hg = 0; hg < NHG; hg++) {
            xs_r[hg] = (wave * HP + 4 * hg + row) * 64 + n;
            xs_rot[hg] = (row + wave * NHG + hg) & 3;
        }
#pragma unroll
        for (int rb = 0; rb < NRB; rb++)
#pragma unroll
            for (int c = 0; c < NCT; c++) accv[rb][c] = v4f{0.0f, 0.0f, 0.0f, 0.0f};
        // the scores of the first two chunks
#pragma unroll
        for (int c0 = 0; c0 < 2; c0++)
            if (c0 < n_chunks) {
                u32x4 kb[NHG][4];
                kmean_fetch(kb, blk_of(c0), c0);
                glb_wait_but<0>();
#pragma unroll
                for (int e = 0; e < NHG; e++)
#pragma unroll
                    for (int ks = 0; ks < 4; ks++) glb_got(kb[e][ks]);
                kmean_scores(kb, c0);
            }
        if (lane < 16) lds_ev[lane] = 0u;
        wave_lds_fence();
        __builtin_amdgcn_s_barrier();
    }
    // The value-mean product of one chunk (it runs after the value side of the next): this wave's strip
    // of the tile, as it came from memory (lane = token), meets everybody's weights and rescale factors
    // of that chunk (exchange buffers, copy sl).  The token index is the contraction index, so the strip
    // is transposed on the way: through the wave's operand scratch, which is free then, a channel tile
    // (2 KiB: [16 channels][64 tokens], the 16-byte groups of a row exchanged by the channel so that the
    // operand reads spread over the banks) at a time; the rows of the scratch that the operand builders
    // rely on as zero are cleared again.  (The LDS reads by hand: the wave's next chunk is on its way
    // into LDS.)
    auto vmean_add_late = [&](const u32x4 (&vm_)[NCT][2], int sl) {
        static_assert(OPER_DW >= 512, "a channel tile of the value-mean strip fits the operand scratch");
        static_assert(NCT <= 2 && NRB <= 2, "operand reads of the value-mean product are written out for these");
        const _Float16 *pb = (const _Float16 *)lds_pb + sl * (2 * HQP * (PB_ROW / 2));
        const float *al = (const float *)lds_al + sl * HQP;
        const uint32_t pba = lds_addr(pb) + n * PB_ROW + 16 * row; // A operand: row n = head n of a block, tokens 8 row .. + 7
        const uint32_t ala = lds_addr(al) + 16 * row;              // factors of heads 4 row .. + 3 of a block
        u32x4 vb[NCT][2], ph[NRB][2], pl[NRB][2], al4[NRB];
        lds_get16<0>(ph[0][0], pba);
        lds_get16<64>(ph[0][1], pba);
        lds_get16<HQP * PB_ROW>(pl[0][0], pba);
        lds_get16<HQP * PB_ROW + 64>(pl[0][1], pba);
        lds_get16<0>(al4[0], ala);
        if (NRB == 2) {
            lds_get16<16 * PB_ROW>(ph[NRB - 1][0], pba);
            lds_get16<16 * PB_ROW + 64>(ph[NRB - 1][1], pba);
            lds_get16<(HQP + 16) * PB_ROW>(pl[NRB - 1][0], pba);
            lds_get16<(HQP + 16) * PB_ROW + 64>(pl[NRB - 1][1], pba);
            lds_get16<64>(al4[NRB - 1], ala);
        }
        lds_wait();
#pragma unroll
        for (int rb = 0; rb < NRB; rb++) { lds_got(ph[rb][0]); lds_got(ph[rb][1]); lds_got(pl[rb][0]); lds_got(pl[rb][1]); lds_got(al4[rb]); }
        unsigned char *vt = (unsigned char *)ak;
        // lane = token on the way in: 16-byte group lane / 8 of a channel's row, exchanged by the channel
        const uint32_t vrd = lds_addr(vt) + n * 128 + ((row ^ (n & 7)) << 4);        // channel n, tokens 8 row .. + 7
        const uint32_t vrd2 = lds_addr(vt) + n * 128 + (((row + 4) ^ (n & 7)) << 4); // ... tokens 32 + 8 row .. + 7
#pragma unroll
        for (int c = 0; c < NCT; c++) {
#pragma unroll
            for (int hf = 0; hf < 2; hf++)
#pragma unroll
                for (int k = 0; k < 4; k++) {
                    const uint32_t w = vm_[c][hf][k];
                    const int ch = 8 * hf + 2 * k;
                    *(uint16_t *)(vt + ch * 128 + (((lane >> 3) ^ (ch & 7)) << 4) + (lane & 7) * 2) = (uint16_t)(w & 0xFFFFu);
                    *(uint16_t *)(vt + (ch + 1) * 128 + (((lane >> 3) ^ ((ch + 1) & 7)) << 4) + (lane & 7) * 2) = (uint16_t)(w >> 16);
                }
            wave_lds_fence();
            lds_get16<0>(vb[c][0], vrd);
            lds_get16<0>(vb[c][1], vrd2);
            lds_wait();
            lds_got(vb[c][0]);
            lds_got(vb[c][1]);
        }
        // words 16 j + 12 .. 15 of the scratch are the fourth limb's rows
#pragma unroll
        for (int j = 0; j < 2; j++) ak[((lane >> 2) + 16 * j) * 16 + 12 + (lane & 3)] = 0u;
#pragma unroll
        for (int rb = 0; rb < NRB; rb++)
#pragma unroll
            for (int c = 0; c < NCT; c++) {
                v4f acc = accv[rb][c] * __builtin_bit_cast(v4f, al4[rb]);
#pragma unroll
                for (int ks = 0; ks < 2; ks++) acc = mfma_h(pl[rb][ks], vb[c][ks], mfma_h(ph[rb][ks], vb[c][ks], acc));
                accv[rb][c] = acc;
            }
    };
    // the strip of the previous chunk, and the copy of the exchange buffers that belongs to the chunk at
    // hand (chunk mod 3)
    u32x4 vmq[NCT][2];
    int xsl = 0;
    const uint32_t eva = lds_addr(lds_ev);

    // cross-head mean: q . mean_K of this lane's tokens (16 k + n of a chunk), worked out by the
    // kernel that ran before this one; loaded one chunk ahead
    long long xq[NHG]; // query head index in the batch
    float xsn[NHG][4];
    auto load_xs = [&](int ci) {
        const int blk = blk_of(ci);
#pragma unroll
        for (int hg = 0; hg < NHG; hg++)
#pragma unroll
            for (int k = 0; k < 4; k++)
                xsn[hg][k] = blk + k / TPB < b_end ? a.xs[xq[hg] * a.tcap + (long long)blk * G + 16 * k + n] : 0.0f;
    };
    if (XH) {
#pragma unroll
        for (int hg = 0; hg < NHG; hg++) {
            const int head = 4 * hg + row;
            xq[hg] = (long long)b * a.n_q_heads + h * g + (head < g ? head : 0);
        }
        if (XH == 1 && wave < n_chunks) load_xs(wave);
    }

    // Issue priority falls as a wave advances (quarters of its chunks).  By default the oldest wave
    // of a SIMD wins every arbitration, so the workgroups that arrived first on a compute unit run
    // ahead and leave the last ones to finish alone, at low occupancy and far below the memory
    // rate; with the laggards preferred, all waves end within about a quarter of each other.
    const int my_iters = (n_chunks - cw0 + CW - 1) / CW;
    PHASE_INIT
    for (int ci = cw0, itn = 0; ci < n_chunks; ci += CW, itn++) {
        PHASE_ITER
        if (KB != 8 || VB != 8) { // the 8-bit instance runs one wave per SIMD: nothing to arbitrate
            const int quart = itn * 4 / my_iters;
            if (quart == 0) __builtin_amdgcn_s_setprio(3);
            else if (quart == 1) __builtin_amdgcn_s_setprio(2);
            else if (quart == 2) __builtin_amdgcn_s_setprio(1);
            else __builtin_amdgcn_s_setprio(0);
        }
        const int blk0 = blk_of(ci);
        bool blk_ok[NBC];
#pragma unroll
        for (int bi = 0; bi < NBC; bi++) blk_ok[bi] = blk0 + bi < b_end;
        // block and tile-in-block of chunk tile `row` (this lane's token group on the value side)
        const unsigned char *sb8 = (const unsigned char *)stage;
        const unsigned char *rec_row = sb8 + (row / TPB) * REC;
        const int tt_row = row % TPB;

        // ---- staged chunk -> registers
        PHASE(0)
        const bool more = ci + CW < n_chunks;
        u32x4 kmB[NHG][4], vmp[NCT][2]; // fused cross-head form: operands fetched by hand
        stage_wait(); // this wave's chunk has landed
        if (XF) {
            // Requested here, ahead of the next chunk's fetch (loads return in order: the wait for
            // these then leaves that fetch alone), and used after the key side, whose arithmetic
            // covers the latency: the key-mean rows of the chunk after the next (of this one again if
            // there is none: the scores are then worked out for nobody), and this wave's strip of this
            // chunk's value-mean tile, lane = token, 32 bytes per channel tile.
            if (PG && itn + 2 - slot_base >= 64) load_slots(itn); // slots of this chunk and the next two
            const bool two_on = ci + 2 * CW < n_chunks;
            kmean_fetch(kmB, two_on ? blk_of(ci + 2 * CW) : blk0, two_on ? itn + 2 : itn);
#pragma unroll
            for (int c = 0; c < NCT; c++)
#pragma unroll
                for (int hf = 0; hf < 2; hf++)
                    glb_get16(vmp[c][hf], mean_row_src(1, blk0, lane, itn) + 32 * (wave * NCT + c) + 16 * hf);
        }
        PHASE(1)
        uint4 kc[NKL], vc[NVL];
#pragma unroll
        for (int i = 0; i < NKL; i++) {
            int bi, off;
            if (KB == 4) { bi = i / TPB; off = (i % TPB) * 64; }
            else if (KB == 2) { bi = (2 * i) / TPB; off = (((2 * i) % TPB) / 2) * 64; }
            else { bi = (i / 2) / TPB; off = (((i / 2) % TPB) * 2 + (i & 1)) * 64; }
            kc[i] = *(const uint4 *)(sb8 + bi * REC + RL::K_CODES + (off + lane) * 16);
        }
#pragma unroll
        for (int i = 0; i < NVL; i++)
            vc[i] = *(const uint4 *)(rec_row + RL::V_CODES + ((i * TPB + tt_row) * 16 + n) * 16);
        uint32_t vm[4][NG];
#pragma unroll
        for (int k = 0; k < 4; k++) {
            const unsigned char *p = sb8 + (k / TPB) * REC + RL::V_META + (((k % TPB) * 16 + n) * NG) * 4;
            if (NG == 4) {
                const uint4 t = *(const uint4 *)p;
                vm[k][0] = t.x; vm[k][1 % NG] = t.y; vm[k][2 % NG] = t.z; vm[k][3 % NG] = t.w;
            } else if (NG == 1) {
                vm[k][0] = *(const uint32_t *)p;
            } else {
                const uint2 t = *(const uint2 *)p;
                vm[k][0] = t.x; vm[k][1 % NG] = t.y;
            }
        }
        uint2 ks[NBC][2], kz[NBC][2], km[NBC][2];
#pragma unroll
        for (int bi = 0; bi < NBC; bi++)
#pragma unroll
            for (int ph = 0; ph < 2; ph++) {
                const int co = (32 * vq + 16 * ph + 4 * qa) * 2;
                ks[bi][ph] = *(const uint2 *)(sb8 + bi * REC + RL::K_SCALE + co);
                kz[bi][ph] = *(const uint2 *)(sb8 + bi * REC + RL::K_ZERO + co);
                km[bi][ph] = MEAN ? *(const uint2 *)(sb8 + bi * REC + RL::K_MEAN + co) : uint2{0u, 0u};
            }
        uint16_t vmean[NBC][8];
#pragma unroll
        for (int bi = 0; bi < NBC; bi++)
#pragma unroll
            for (int ct = 0; ct < 8; ct++)
                vmean[bi][ct] = MEAN ? *(const uint16_t *)(sb8 + bi * REC + RL::V_MEAN + (16 * ct + n) * 2) : (uint16_t)0;
        // The mean's scores of this chunk are taken over, and those of the next chunk requested,
        // before the next chunk's fetch is issued: loads return in order, and the compiler, which
        // cannot see the wait above, would otherwise wait for everything outstanding -- the fetch
        // just issued included -- before it lets the registers of the previous request be reused.
        float xsv[NHG][4];
        long long xbase[NHG]; // this lane's first token of the chunk in xs / xp
        if (XH == 1) {
#pragma unroll
            for (int hg = 0; hg < NHG; hg++) {
                xbase[hg] = xq[hg] * a.tcap + (long long)blk0 * G;
#pragma unroll
                for (int k = 0; k < 4; k++) xsv[hg][k] = xsn[hg][k];
            }
            if (ci + NW < n_chunks) load_xs(ci + NW);
        }
        // every read of the staging buffer has returned: start fetching this wave's next chunk
        wave_lds_fence();
        if (more) issue(ci + CW);
        PHASE(2)
        if (XF) {
            // q . mean_K of token 16 k + n for head `row` of each head group, worked out by the waves
            // together during the previous chunk
            const float *xs = (const float *)lds_xs + xsl * (HQP * 64);
#pragma unroll
            for (int hg = 0; hg < NHG; hg++)
#pragma unroll
                for (int k = 0; k < 4; k++) xsv[hg][k] = xs[xs_r[hg] + (((k + xs_rot[hg]) & 3) << 4)];
        }

        // ---- key side, one block at a time (the operand scratch holds one block's operands):
        // q*scale as limbs -> LDS, zero/mean term, then the block's matrix products -> scores
        float s[NHG][4];
#pragma unroll
        for (int bi = 0; bi < NBC; bi++) {
            // scales are non-negative binary16 values: their bit patterns order like the values,
            // so the largest is found with packed 16-bit integer maxima on the raw words
            uint32_t smw = pk_max_u16(pk_max_u16(ks[bi][0].x, ks[bi][0].y), pk_max_u16(ks[bi][1].x, ks[bi][1].y));
            smw = row_pk_max_u16(smw);
            const float sb = pow2_above_h2(smw, true);
            float inv_kf[NHG], beta[NHG];
#pragma unroll
            for (int hg = 0; hg < NHG; hg++) {
                inv_kf[hg] = inv_kf_base[hg] * sb;
                // Adding 3 qb sb (1.5 * 2^E with 2^E = 2 qb sb > 2 |q s|) puts round(q s / ulp) into
                // the low mantissa bits of the sum, ulp = qb sb 2^-22: one fused multiply-add per
                // element does the scaling, the rounding and the float -> integer conversion.
                const float magic = three_qb[hg] * sb;
                const uint32_t cfix = opaque(0x80808080u - __float_as_uint(magic));
                float bacc = 0.0f;
#pragma unroll
                for (int ph = 0; ph < 2; ph++) {
                    uint32_t X[4];
#pragma unroll
                    for (int y = 0; y < 4; y++) {
                        const uint32_t sw = (y & 2) ? ks[bi][ph].y : ks[bi][ph].x;
                        const float sv = (y & 1) ? h_hi(sw) : h_lo(sw);
                        X[y] = __float_as_uint(__builtin_fmaf(qf[hg][ph][y], sv, magic)) + cfix;
                    }
                    // 4 x 4 byte transpose: limb L of the lane's four consecutive channels
                    const uint32_t U = __builtin_amdgcn_perm(X[1], X[0], 0x05010400u);
                    const uint32_t U2 = __builtin_amdgcn_perm(X[1], X[0], 0x07030602u);
                    const uint32_t W = __builtin_amdgcn_perm(X[3], X[2], 0x05010400u);
                    const uint32_t W2 = __builtin_amdgcn_perm(X[3], X[2], 0x07030602u);
                    const uint32_t Y0 = __builtin_amdgcn_perm(W, U, 0x05040100u);
                    const uint32_t Y1 = __builtin_amdgcn_perm(W, U, 0x07060302u);
                    const uint32_t Y2 = __builtin_amdgcn_perm(W2, U2, 0x05040100u);
                    uint32_t *dst = ak + hg * 512 + ((ph * 4 + vq) * 16 + 4 * row) * 4 + qa;
                    // biased bytes -> signed bytes, after the transpose (three words instead of four)
                    dst[0] = Y0 ^ 0x80808080u;
                    dst[4] = Y1 ^ 0x80808080u;
                    dst[8] = Y2 ^ 0x80808080u;
                    bacc = __builtin_amdgcn_fdot2(qh[hg][ph][0], as_h2(kz[bi][ph].x), bacc, false);
                    bacc = __builtin_amdgcn_fdot2(qh[hg][ph][1], as_h2(kz[bi][ph].y), bacc, false);
                    bacc = __builtin_amdgcn_fdot2(qh[hg][ph][0], as_h2(km[bi][ph].x), bacc, false);
                    bacc = __builtin_amdgcn_fdot2(qh[hg][ph][1], as_h2(km[bi][ph].y), bacc, false);
                }
                beta[hg] = row_sum(bacc) * kScoreScale;
            }
            wave_lds_fence();
            v4i a0[NHG], a1[NHG];
#pragma unroll
            for (int hg = 0; hg < NHG; hg++) {
                a0[hg] = *(const v4i *)(ak + hg * 512 + ((0 * 4 + row) * 16 + n) * 4);
                a1[hg] = *(const v4i *)(ak + hg * 512 + ((1 * 4 + row) * 16 + n) * 4);
            }
            wave_lds_fence(); // the operands are in registers: the scratch may be overwritten
#pragma unroll
            for (int k = bi * TPB; k < (bi + 1) * TPB; k++) {
                v4i acc[NHG];
                if (KB == 4) {
                    const uint4 w = kc[k];
                    const v4i b0 = CodeOps<4>::line(w.x, w.y), b1 = CodeOps<4>::line(w.z, w.w);
#pragma unroll
                    for (int hg = 0; hg < NHG; hg++) acc[hg] = mfma(a1[hg], b1, mfma(a0[hg], b0, v4i{0, 0, 0, 0}));
                } else if (KB == 2) {
                    const uint4 w = kc[k >> 1];
                    const v4i b0 = CodeOps<2>::line((k & 1) ? w.z : w.x), b1 = CodeOps<2>::line((k & 1) ? w.w : w.y);
#pragma unroll
                    for (int hg = 0; hg < NHG; hg++) acc[hg] = mfma(a1[hg], b1, mfma(a0[hg], b0, v4i{0, 0, 0, 0}));
                } else {
                    const uint4 wa = kc[2 * k], wb = kc[2 * k + 1];
                    const v4i lo0 = CodeOps<8>::lo(wa), hi0 = CodeOps<8>::hi(wa);
                    const v4i lo1 = CodeOps<8>::lo(wb), hi1 = CodeOps<8>::hi(wb);
#pragma unroll
                    for (int hg = 0; hg < NHG; hg++) {
                        const v4i alo = mfma(a1[hg], lo1, mfma(a0[hg], lo0, v4i{0, 0, 0, 0}));
                        const v4i ahi = mfma(a1[hg], hi1, mfma(a0[hg], hi0, v4i{0, 0, 0, 0}));
                        acc[hg] = alo + ahi * 16;
                    }
                }
#pragma unroll
                for (int hg = 0; hg < NHG; hg++) {
                    float sc_ = limbs_to_float(acc[hg]) * inv_kf[hg] + beta[hg];
                    if (XH) sc_ += xsv[hg][k] * kScoreScale;
                    s[hg][k] = blk_ok[bi] ? sc_ : -INFINITY;
                }
            }
        }

        PHASE(5)
        // ---- largest value scale of the chunk (the same for every head)
        uint32_t svw = 0u; // low halves: scales (high halves, the zeros, are ignored)
#pragma unroll
        for (int k = 0; k < 4; k++)
#pragma unroll
            for (int gam = 0; gam < NG; gam++) svw = pk_max_u16(svw, vm[k][gam]);
        svw = row_pk_max_u16(svw);
        const float sbv = pow2_above_h2(svw, false);
        const float vmagic = 3.0f * sbv; // p <= 1, scale < sbv: same construction as on the key side
        const uint32_t vfix = opaque(0x80808080u - __float_as_uint(vmagic));

        // ---- softmax bookkeeping; zero and mean terms of the value side
        float p[NHG][4], alpha[NHG], o_scale[NHG], psum_b[NHG][NBC], wcs[NHG];
#pragma unroll
        for (int hg = 0; hg < NHG; hg++) {
            float wc, mc;
            softmax_chunk(s[hg], st[hg], p[hg], alpha[hg], wc, mc);
            wcs[hg] = wc;
            if (XH == 1 && 4 * hg + row < g) {
                // the weights and the chunk's maximum, for the value mean plane's share
#pragma unroll
                for (int k = 0; k < 4; k++)
                    if (blk_ok[k / TPB]) a.xp[xbase[hg] + 16 * k + n] = p[hg][k];
                if (n == 0) a.xmc[xq[hg] * (a.tcap / 64 + 1) + blk0 / NBC] = mc;
            }
            o_scale[hg] = wc * sbv * 0x1p-22f;
#pragma unroll
            for (int gam = 0; gam < NG; gam++) {
                float zsum = 0.0f;
#pragma unroll
                for (int k = 0; k < 4; k++) zsum += p[hg][k] * h_hi(vm[k][gam]);
                st[hg].Zp[gam] = st[hg].Zp[gam] * alpha[hg] + wc * zsum;
            }
#pragma unroll
            for (int bi = 0; bi < NBC; bi++) {
                float t = 0.0f;
#pragma unroll
                for (int k = bi * TPB; k < (bi + 1) * TPB; k++) t += p[hg][k];
                psum_b[hg][bi] = MEAN ? row_sum(t) * wc : 0.0f;
            }
        }

        // ---- fused cross-head form: the value mean's share, sum_t p_t mean_V[t], for all heads of the
        // workgroup and this wave's channel tile(s), kept relative to each head's running maximum
        PHASE(6)
        if (XF) {
            // this wave's weights, relative to the new running maximum and times 2^8 (so that the low
            // part of a small weight is still a normal binary16 number), as binary16 hi + lo; and the
            // factor that brings the old sums to the new maximum
            _Float16 *pb = (_Float16 *)lds_pb + xsl * (2 * HQP * (PB_ROW / 2));
            float *al = (float *)lds_al + xsl * HQP;
#pragma unroll
            for (int hg = 0; hg < NHG; hg++) {
                const int hp = wave * HP + 4 * hg + row;
#pragma unroll
                for (int k = 0; k < 4; k++) {
                    const float pv = p[hg][k] * (wcs[hg] * 256.0f);
                    const _Float16 hi = (_Float16)pv;
                    pb[hp * (PB_ROW / 2) + 16 * k + n] = hi;
                    pb[(HQP + hp) * (PB_ROW / 2) + 16 * k + n] = (_Float16)(pv - (float)hi);
                }
                if (n == 0) al[hp] = alpha[hg];
            }
            PHASE(7)
            // the operands fetched by hand are there (fetches issued since: the next chunk, if any)
            constexpr int nCmin = NBC == 1 ? (CB + 1023) / 1024
                                           : ((CB + 1023) / 1024 < 2 * ((REC + 1023) / 1024) ? (CB + 1023) / 1024 : 2 * ((REC + 1023) / 1024));
            if (more) glb_wait_but<nCmin>();
            else glb_wait_but<0>();
#pragma unroll
            for (int e = 0; e < NHG; e++)
#pragma unroll
                for (int ks = 0; ks < 4; ks++) glb_got(kmB[e][ks]);
#pragma unroll
            for (int c = 0; c < NCT; c++)
#pragma unroll
                for (int hf = 0; hf < 2; hf++) glb_got(vmp[c][hf]);
        }

        // ---- value side in passes of NGP scale groups: p*scale as limbs -> LDS, matrix products
        // -> output accumulators
#pragma unroll
        for (int vp = 0; vp < NG / NGP; vp++) {
#pragma unroll
            for (int hg = 0; hg < NHG; hg++)
#pragma unroll
                for (int gl = 0; gl < NGP; gl++) {
                    const int gam = vp * NGP + gl;
#pragma unroll
                    for (int k = 0; k < 4; k++) {
                        const uint32_t X = (__float_as_uint(__builtin_fmaf(p[hg][k], h_lo(vm[k][gam]), vmagic)) + vfix) ^ 0x80808080u;
                        // limb L of token 4 vq + qa of tile k is byte qa of word (4 row + L) * 4 + vq:
                        // three byte stores (the LDS port is idle, the vector ALU is not)
                        unsigned char *o8 = (unsigned char *)(av + (hg * NGP + gl) * 256 + k * 64 + (4 * row) * 4 + vq) + qa;
                        o8[0] = (unsigned char)X;
                        o8[16] = (unsigned char)(X >> 8);
                        o8[32] = (unsigned char)(X >> 16);
                    }
                }
            wave_lds_fence();
            v4i avr[NHG][NGP];
#pragma unroll
            for (int hg = 0; hg < NHG; hg++)
#pragma unroll
                for (int gl = 0; gl < NGP; gl++)
                    avr[hg][gl] = *(const v4i *)(av + (hg * NGP + gl) * 256 + (row * 16 + n) * 4);
            wave_lds_fence(); // operands in registers: the next pass (or chunk) may overwrite the scratch
#pragma unroll
            for (int ct = vp * NGP * TPG; ct < (vp + 1) * NGP * TPG; ct++) {
                const int gl = ct / TPG - vp * NGP;
                v4i acc[NHG];
                if (VB == 4) {
                    const uint4 w = vc[ct >> 1];
                    const v4i bo = CodeOps<4>::line((ct & 1) ? w.z : w.x, (ct & 1) ? w.w : w.y);
#pragma unroll
                    for (int hg = 0; hg < NHG; hg++) acc[hg] = mfma(avr[hg][gl], bo, v4i{0, 0, 0, 0});
                } else if (VB == 2) {
                    const uint4 w = vc[ct >> 2];
                    const uint32_t ww = (ct & 3) == 0 ? w.x : ((ct & 3) == 1 ? w.y : ((ct & 3) == 2 ? w.z : w.w));
                    const v4i bo = CodeOps<2>::line(ww);
#pragma unroll
                    for (int hg = 0; hg < NHG; hg++) acc[hg] = mfma(avr[hg][gl], bo, v4i{0, 0, 0, 0});
                } else {
                    const v4i lo = CodeOps<8>::lo(vc[ct]), hi = CodeOps<8>::hi(vc[ct]);
#pragma unroll
                    for (int hg = 0; hg < NHG; hg++) {
                        const v4i alo = mfma(avr[hg][gl], lo, v4i{0, 0, 0, 0});
                        const v4i ahi = mfma(avr[hg][gl], hi, v4i{0, 0, 0, 0});
                        acc[hg] = alo + ahi * 16;
                    }
                }
#pragma unroll
                for (int hg = 0; hg < NHG; hg++) {
                    float o = st[hg].O[ct] * alpha[hg] + limbs_to_float(acc[hg]) * o_scale[hg];
#pragma unroll
                    for (int bi = 0; bi < NBC; bi++)
                        o += __half2float(__ushort_as_half(vmean[bi][ct])) * psum_b[hg][bi];
                    st[hg].O[ct] = o;
                }
            }
        }
        if (XF) {
            // (a wave's counter = the chunks it has finished) the product of the PREVIOUS
            // chunk, once every wave has finished that chunk -- its weights and factors, written half a
            // chunk ago at the latest, are then in place --, and the scores of the chunk after the next
            // into the copy whose scores (of the previous chunk) everybody has then read.  A copy is
            // written again three chunks later, and no wave gets more than one chunk ahead of another.
            if (itn > 0) {
                progress_wait_all<NW>(eva, (uint32_t)itn, lane);
                vmean_add_late(vmq, xsl == 0 ? 2 : xsl - 1);
            }
            kmean_scores(kmB, xsl == 0 ? 2 : xsl - 1);
#pragma unroll
            for (int c = 0; c < NCT; c++) { vmq[c][0] = vmp[c][0]; vmq[c][1] = vmp[c][1]; }
            progress_publish(eva + 4 * wave, (uint32_t)itn + 1u, lane);
            xsl = xsl == 2 ? 0 : xsl + 1;
        }
        PHASE(11)
    }
    PHASE(12)

    if (KB != 8 || VB != 8) __builtin_amdgcn_s_setprio(0);

    // fused cross-head form: the value mean's share goes from the waves that summed it (all heads, a
    // channel tile) to the waves that own the heads, through the buffer the scores went through
    if (XF) {
        {
            __builtin_amdgcn_s_barrier(); // (everybody has left the loop: a barrier serves)
            if (n_chunks > 0) vmean_add_late(vmq, xsl == 0 ? 2 : xsl - 1); // the last chunk's product
        }
        float *om = (float *)lds_xs; // [head][128]
#pragma unroll
        for (int rb = 0; rb < NRB; rb++)
#pragma unroll
            for (int c = 0; c < NCT; c++)
#pragma unroll
                for (int j = 0; j < 4; j++)
                    om[(16 * rb + 4 * row + j) * kHeadDim + 16 * (wave * NCT + c) + n] = accv[rb][c][j] * 0x1p-8f;
        __syncthreads();
#pragma unroll
        for (int hg = 0; hg < NHG; hg++)
#pragma unroll
            for (int ct = 0; ct < 8; ct++) st[hg].O[ct] += om[(wave * HP + 4 * hg + row) * kHeadDim + 16 * ct + n];
    }

    // ---- raw residual tokens (Sec. 3.3) in tiles of 32, dealt to the splits in turn after the
    // unit's last chunk; wave w of the split takes tokens 8 w .. 8 w + 7 of a tile into its own
    // online-softmax state, with its own LDS region as scratch (no workgroup barrier)
    const int rt_first = (sp - chunks_total % ns + ns) % ns; // this split's first tile
    if (rt_first * 32 + 8 * cw0 < r_seq) {
        unsigned char *L = (unsigned char *)lds;
        constexpr int RS = 264;  // bytes per staged row (33 * 8): rows start in different banks
        constexpr int NH = 4 * NHG;
        unsigned char *kraw = L, *vraw = L + 8 * RS;
        uint16_t *qs = (uint16_t *)(L + 16 * RS);             // [NH][128], the queries as they came
        float *spart = (float *)(L + 16 * RS + NH * 256);      // [8 channel slices][NH][8 tokens]
        float *pl = spart + 8 * NH * 8;                        // [NH][8]
        static_assert(16 * RS + NH * 256 + (8 * NH * 8 + NH * 8) * 4 <= WAVE_DW * 4, "residual scratch");
        wave_lds_fence();
#pragma unroll
        for (int hg = 0; hg < NHG; hg++)
#pragma unroll
            for (int ph = 0; ph < 2; ph++)
#pragma unroll
                for (int y = 0; y < 4; y++) {
                    // narrowing a widened 16-bit value is exact
                    const float qv = qf[hg][ph][y];
                    const uint16_t q16 = gm.dtype == 1 ? (uint16_t)(__float_as_uint(qv) >> 16)
                                                       : __half_as_ushort(__float2half_rn(qv));
                    qs[(4 * hg + row) * 128 + 32 * vq + 16 * ph + 4 * qa + y] = q16;
                }
        const unsigned char *kr = a.layer + gm.k_resid_off + (long long)u * gm.R * 256;
        const unsigned char *vr = a.layer + gm.v_resid_off + (long long)u * gm.R * 256;
        // a token appended by this very call: read from the caller's rows and stored in the cache here
        const long long fresh_off = (long long)b * a.fresh_stride_b + (long long)h * a.fresh_stride_h;
        const int t_fresh = a.k_fresh ? r_seq - 1 : -1;
        // (fused cross-head form: the wave has the unit to itself and takes all four groups of a tile)
        for (int tg8 = XF ? 0 : wave;; tg8 += XF ? 1 : 4) {
            const int t0 = (rt_first + ns * (tg8 >> 2)) * 32 + 8 * (tg8 & 3);
            if ((rt_first + ns * (tg8 >> 2)) * 32 >= r_seq) break;
            if (t0 >= r_seq) continue;
            const int nt = r_seq - t0 < 8 ? r_seq - t0 : 8;
            wave_lds_fence();
            for (int i = lane; i < nt * 16; i += 64) {
                const int t = i >> 4, ch = i & 15;
                uint4 kv_, vv_;
                if (t0 + t == t_fresh) {
                    kv_ = *(const uint4 *)(a.k_fresh + fresh_off + ch * 8);
                    vv_ = *(const uint4 *)(a.v_fresh + fresh_off + ch * 8);
                    *(uint4 *)const_cast<unsigned char *>(kr + (long long)t_fresh * 256 + ch * 16) = kv_;
                    *(uint4 *)const_cast<unsigned char *>(vr + (long long)t_fresh * 256 + ch * 16) = vv_;
                } else {
                    kv_ = *(const uint4 *)(kr + (long long)(t0 + t) * 256 + ch * 16);
                    vv_ = *(const uint4 *)(vr + (long long)(t0 + t) * 256 + ch * 16);
                }
                *(uint2 *)(kraw + t * RS + ch * 16) = uint2{kv_.x, kv_.y};
                *(uint2 *)(kraw + t * RS + ch * 16 + 8) = uint2{kv_.z, kv_.w};
                *(uint2 *)(vraw + t * RS + ch * 16) = uint2{vv_.x, vv_.y};
                *(uint2 *)(vraw + t * RS + ch * 16 + 8) = uint2{vv_.z, vv_.w};
            }
            wave_lds_fence();
            {
                // lane (token t, slice sl): q . k over channels 16 sl .. 16 sl + 15, every head
                const int t = lane & 7, sl = lane >> 3;
                float dn[NH];
#pragma unroll
                for (int i = 0; i < NH; i++) dn[i] = 0.0f;
                if (t < nt) {
#pragma unroll
                    for (int c = 0; c < 16; c += 2) {
                        const uint32_t w = *(const uint32_t *)(kraw + t * RS + (16 * sl + c) * 2);
                        const float k0 = widen16((uint16_t)(w & 0xFFFFu), gm.dtype);
                        const float k1 = widen16((uint16_t)(w >> 16), gm.dtype);
#pragma unroll
                        for (int i = 0; i < NH; i++) {
                            const uint32_t qw = *(const uint32_t *)(qs + i * 128 + 16 * sl + c);
                            dn[i] += widen16((uint16_t)(qw & 0xFFFFu), gm.dtype) * k0 + widen16((uint16_t)(qw >> 16), gm.dtype) * k1;
                        }
                    }
                }
#pragma unroll
                for (int i = 0; i < NH; i++) spart[(sl * NH + i) * 8 + t] = dn[i];
            }
            wave_lds_fence();
            float pr[NHG], al[NHG], wcr[NHG];
#pragma unroll
            for (int hg = 0; hg < NHG; hg++) {
                const int head = 4 * hg + row;
                float s[4], p[4];
                float dot = 0.0f;
#pragma unroll
                for (int sl = 0; sl < 8; sl++) dot += spart[(sl * NH + head) * 8 + (n & 7)];
                s[0] = n < nt ? dot * kScoreScale : -INFINITY;
                s[1] = s[2] = s[3] = -INFINITY;
                float mcr;
                softmax_chunk(s, st[hg], p, al[hg], wcr[hg], mcr);
                pr[hg] = p[0];
            }
#pragma unroll
            for (int hg = 0; hg < NHG; hg++)
                if (n < nt) pl[(4 * hg + row) * 8 + n] = pr[hg];
            wave_lds_fence();
#pragma unroll
            for (int hg = 0; hg < NHG; hg++) {
                float add[8];
#pragma unroll
                for (int ct = 0; ct < 8; ct++) add[ct] = 0.0f;
                for (int t = 0; t < nt; t++) {
                    const float pv = pl[(4 * hg + row) * 8 + t];
#pragma unroll
                    for (int ct = 0; ct < 8; ct++)
                        add[ct] += pv * widen16(*(const uint16_t *)(vraw + t * RS + (16 * ct + n) * 2), gm.dtype);
                }
#pragma unroll
                for (int ct = 0; ct < 8; ct++) st[hg].O[ct] = st[hg].O[ct] * al[hg] + wcr[hg] * add[ct];
#pragma unroll
                for (int gam = 0; gam < 4; gam++) st[hg].Zp[gam] *= al[hg];
            }
        }
    }

    // ---- finish the wave's state and merge the waves: [NHG][10][64] floats at the start of each wave's LDS
    static_assert(NHG * 10 * 64 <= WAVE_DW, "state exchange");
    float *mine = (float *)lds;
    wave_lds_fence();
#pragma unroll
    for (int hg = 0; hg < NHG; hg++) {
        st[hg].l = row_sum(st[hg].l);
#pragma unroll
        for (int gam = 0; gam < NG; gam++) {
            const float z = row_sum(st[hg].Zp[gam]);
#pragma unroll
            for (int ct = gam * TPG; ct < (gam + 1) * TPG; ct++) st[hg].O[ct] += z;
        }
        mine[(hg * 10 + 0) * 64 + lane] = st[hg].M;
        mine[(hg * 10 + 1) * 64 + lane] = st[hg].l;
#pragma unroll
        for (int ct = 0; ct < 8; ct++) mine[(hg * 10 + 2 + ct) * 64 + lane] = st[hg].O[ct];
    }
    PHASE(13)
    PHASE_DONE
    __syncthreads();
    if (XF || wave == 0) {
        constexpr int MW = XF ? 1 : NW; // waves whose states make up the partial result
        const float *all = (const float *)lds_all + (XF ? wave * WAVE_DW : 0);
#pragma unroll
        for (int hg = 0; hg < NHG; hg++) {
            const int head = 4 * hg + row;
            if (head >= g) continue;
            float Mw[MW], M = -INFINITY;
#pragma unroll
            for (int w = 0; w < MW; w++) {
                Mw[w] = all[w * WAVE_DW + (hg * 10 + 0) * 64 + lane];
                M = fmaxf(M, Mw[w]);
            }
            float lsum = 0.0f, o[8];
#pragma unroll
            for (int ct = 0; ct < 8; ct++) o[ct] = 0.0f;
#pragma unroll
            for (int w = 0; w < MW; w++) {
                const float wt = Mw[w] == -INFINITY ? 0.0f : exp2f(Mw[w] - M); // a wave that saw no token
                lsum += all[w * WAVE_DW + (hg * 10 + 1) * 64 + lane] * wt;
#pragma unroll
                for (int ct = 0; ct < 8; ct++) o[ct] += all[w * WAVE_DW + (hg * 10 + 2 + ct) * 64 + lane] * wt;
            }
            float *dst = a.ws + (((long long)u * g + head) * a.n_splits + sp) * kPartialStride;
#pragma unroll
            for (int ct = 0; ct < 8; ct++) dst[16 * ct + n] = o[ct];
            if (n == 0) {
                dst[kHeadDim] = M;
                dst[kHeadDim + 1] = lsum;
            }
        }
    }
}

// Resident workgroups of one instantiation on the whole device (0 if the query fails).
template <int B, int G, int GC, bool MEAN, int NW, int NHG, int XH, bool PG> int resident_blocks()
{
    static const int n = [] {
        int per_cu = 0, dev = 0, cus = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, decode_split_mfma_kernel<B, G, GC, MEAN, NW, NHG, XH, PG>,
                                                         64 * NW, 0) != hipSuccess)
            return 0;
        if (hipGetDevice(&dev) != hipSuccess) return 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
        return per_cu * cus;
    }();
    return n;
}

// Events that the calling thread's next split launch records its own begin and end into (set_split_timing_events)
thread_local hipEvent_t t_ev_begin = nullptr, t_ev_end = nullptr;

// XH == 2 (both cross-head mean terms inside the kernel): a workgroup per (sequence, split) and NW kv heads.
template <int B, int G, int GC, bool MEAN, int NW, int NHG, int XH, bool PG> hipError_t launch_inst(const DecodeArgs &a, hipStream_t s)
{
    if (!RecLayout<B, G, GC, MEAN>::matches(a.geom)) return hipErrorInvalidValue;
    if (XH == 2 && (a.n_kv_heads < NW || a.n_kv_heads % NW != 0)) return hipErrorInvalidValue;
    dim3 grid(XH == 2 ? a.n_splits * (a.n_kv_heads / NW) : a.n_splits, XH == 2 ? a.batch : a.batch * a.n_kv_heads);
    (void)hipGetLastError(); // drop any stale error left by earlier runtime calls of this thread
    if (t_ev_begin && t_ev_end) {
        // the dispatch itself stamps the events: the kernel's execution, without the gaps before and after it
        hipExtLaunchKernelGGL((decode_split_mfma_kernel<B, G, GC, MEAN, NW, NHG, XH, PG>), grid, dim3(64 * NW), 0, s, t_ev_begin,
                              t_ev_end, 0, a);
        t_ev_begin = t_ev_end = nullptr;
    } else {
        hipLaunchKernelGGL((decode_split_mfma_kernel<B, G, GC, MEAN, NW, NHG, XH, PG>), grid, dim3(64 * NW), 0, s, a);
    }
    return note_launch(hipGetLastError());
}

// Split count that puts every workgroup of the launch on the device at once (one "round"):
// the kernel is a bandwidth stream, and a second, partly filled round only adds a tail.
template <int B, int G, int GC, bool MEAN, int NW, int NHG, int XH, bool PG> int plan_inst(const DecodeArgs &a)
{
    const int slots = resident_blocks<B, G, GC, MEAN, NW, NHG, XH, PG>();
    const int U = XH == 2 ? a.batch * (a.n_kv_heads / NW) : a.batch * a.n_kv_heads; // workgroups per split
    constexpr int CW = XH == 2 ? 1 : NW;                      // waves that share a unit's chunks
    const int chunks = (a.n_blocks * G + 63) / 64; // chunks of 64 tokens
    int ns = slots / U;
    // at least four chunks per wave, or the prologue dominates -- unless the launch is so small that
    // the device cannot be filled even then: such a launch is bound by latency, and the widest
    // spread (one chunk per wave) is the shortest
    const bool small = (long long)U * chunks < (long long)slots * CW * 4;
    const int cap = small ? (chunks + CW - 1) / CW : chunks / (CW * 4);
    if (ns > cap) ns = cap;
    if (ns > kMaxSplits) ns = kMaxSplits;
    if (ns < 1) ns = 1;
    return ns;
}

// what to do with the instance selected by the layer's format
struct DoLaunch {
    hipStream_t s;
    hipError_t result = hipErrorInvalidValue;
    template <int B, int G, int GC, bool MEAN, int NW, int NHG, int XH, bool PG> void run(const DecodeArgs &a) { result = launch_inst<B, G, GC, MEAN, NW, NHG, XH, PG>(a, s); }
};
struct DoPlan {
    int result = 1;
    template <int B, int G, int GC, bool MEAN, int NW, int NHG, int XH, bool PG> void run(const DecodeArgs &a) { result = plan_inst<B, G, GC, MEAN, NW, NHG, XH, PG>(a); }
};
struct DoMatch {
    bool result = false;
    template <int B, int G, int GC, bool MEAN, int NW, int NHG, int XH, bool PG> void run(const DecodeArgs &a) { result = RecLayout<B, G, GC, MEAN>::matches(a.geom); }
};

// Does the layer get the fused cross-head form (both mean terms inside the split kernel)?  It takes a
// wave per kv head, a multiple of 4 kv heads.
bool xhead_fused_fmt(const DecodeArgs &a)
{
    const LayerGeom &g = a.geom;
    return g.mean_mode == 1 && a.n_kv_heads % 4 == 0;
}

template <int B, int G, int GC, bool PG, class F> void pick_mean_heads_pg(const DecodeArgs &a, F &f)
{
    constexpr int NW = kWavesPerBlock;
    const int mode = a.geom.mean_mode; // 0 per-channel block mean, 1 cross-head mean, 2 none
    // (the cross-head forms exist for equal group sizes only: decode_mfma_supported)
    if (a.g <= 4) {
        if (mode == 0) f.template run<B, G, GC, true, NW, 1, 0, PG>(a);
        else if (mode == 1) { if constexpr (G == GC && B < 16) f.template run<B, G, GC, false, NW, 1, 1, PG>(a); }
        else f.template run<B, G, GC, false, NW, 1, 0, PG>(a);
    } else {
        if (mode == 0) f.template run<B, G, GC, true, NW, 2, 0, PG>(a);
        else if (mode == 1) { if constexpr (G == GC && B < 16) f.template run<B, G, GC, false, NW, 2, 1, PG>(a); }
        else f.template run<B, G, GC, false, NW, 2, 0, PG>(a);
    }
}
// the fused cross-head instances: a wave per kv head.  Eight kv heads go to two workgroups of four waves
// that share a sequence's split, except at 4 bits with up to four query heads per kv head, where one
// workgroup of eight is faster (177 against 193 us per layer on 16 sequences of 32768 tokens: every
// mean row is fetched once per workgroup instead of once per pair that may have drifted apart in the
// L2; at 2 bits the four-wave instance fits a compute unit twice and wins, 158 against 163 us; eight
// 8-bit chunk buffers do not fit the LDS).
template <int B, int G, int GC, bool PG, class F> void pick_fused_pg(const DecodeArgs &a, F &f)
{
    if constexpr (B == 4) {
        if (a.n_kv_heads % 8 == 0 && a.g <= 4) {
            f.template run<B, G, GC, false, 8, 1, 2, PG>(a);
            return;
        }
    }
    if (a.g <= 4) f.template run<B, G, GC, false, 4, 1, 2, PG>(a);
    else f.template run<B, G, GC, false, 4, 2, 2, PG>(a);
}
template <int B, int G, int GC, class F> void pick_fused(const DecodeArgs &a, F &f)
{
    if (a.geom.table) pick_fused_pg<B, G, GC, true>(a, f);
    else pick_fused_pg<B, G, GC, false>(a, f);
}
template <int B, int G, int GC, class F> void pick_mean_heads(const DecodeArgs &a, F &f)
{
    if (a.geom.table) pick_mean_heads_pg<B, G, GC, true>(a, f);
    else pick_mean_heads_pg<B, G, GC, false>(a, f);
}

template <class F> void pick(const DecodeArgs &a, F &f)
{
    const int bits = a.geom.k_bits;
    if (xhead_fused_fmt(a)) {
        if (a.geom.G == 32) {
            if (bits == 2) pick_fused<2, 32, 32>(a, f);
            else if (bits == 4) pick_fused<4, 32, 32>(a, f);
            else pick_fused<8, 32, 32>(a, f);
        } else if (a.geom.G == 64) {
            if (bits == 2) pick_fused<2, 64, 64>(a, f);
            else if (bits == 4) pick_fused<4, 64, 64>(a, f);
            else pick_fused<8, 64, 64>(a, f);
        } else {
            if (bits == 2) pick_fused<2, 128, 128>(a, f);
            else if (bits == 4) pick_fused<4, 128, 128>(a, f);
            else pick_fused<8, 128, 128>(a, f);
        }
        return;
    }
    if (a.geom.k_bits != a.geom.v_bits) {
        // keys and values of different widths: groups of 32 tokens / 32 channels
        const int kb = a.geom.k_bits, vb = a.geom.v_bits;
        // (dense placement only: the paged instances of six more width pairs are not worth their compile time)
        if (kb == 2 && vb == 4) pick_mean_heads_pg<2 | 4 << 4, 32, 32, false>(a, f);
        else if (kb == 2 && vb == 8) pick_mean_heads_pg<2 | 8 << 4, 32, 32, false>(a, f);
        else if (kb == 4 && vb == 2) pick_mean_heads_pg<4 | 2 << 4, 32, 32, false>(a, f);
        else if (kb == 4 && vb == 8) pick_mean_heads_pg<4 | 8 << 4, 32, 32, false>(a, f);
        else if (kb == 8 && vb == 2) pick_mean_heads_pg<8 | 2 << 4, 32, 32, false>(a, f);
        else pick_mean_heads_pg<8 | 4 << 4, 32, 32, false>(a, f);
        return;
    }
    // every pair (tokens per key group, channels per value group) of 32, 64, 128
#define TADAKV_PICK(GV, GCV)                                      \
    if (a.geom.G == GV && a.geom.Gc == GCV) {                     \
        if (bits == 2) pick_mean_heads<2, GV, GCV>(a, f);         \
        else if (bits == 4) pick_mean_heads<4, GV, GCV>(a, f);    \
        else pick_mean_heads<8, GV, GCV>(a, f);                   \
        return;                                                   \
    }
    TADAKV_PICK(32, 32)
    TADAKV_PICK(64, 64)
    TADAKV_PICK(128, 128)
    TADAKV_PICK(32, 64)
    TADAKV_PICK(32, 128)
    TADAKV_PICK(64, 32)
    TADAKV_PICK(64, 128)
    TADAKV_PICK(128, 32)
    TADAKV_PICK(128, 64)
#undef TADAKV_PICK
}

} // namespace

bool xhead_fused(const DecodeArgs &a) { return decode_mfma_supported(a) && xhead_fused_fmt(a); }

bool decode_mfma_supported(const DecodeArgs &a)
{
    const LayerGeom &g = a.geom;
    if (!(g.k_bits == 2 || g.k_bits == 4 || g.k_bits == 8) || !(g.v_bits == 2 || g.v_bits == 4 || g.v_bits == 8)) return false;
    if (g.k_bits != g.v_bits && !(g.G == 32 && g.Gc == 32 && g.mean_mode != 1 && g.table == nullptr)) return false; // different widths: one format, dense
    const bool sizes = (g.G == 32 || g.G == 64 || g.G == 128) && (g.Gc == 32 || g.Gc == 64 || g.Gc == 128);
    if (!sizes) return false;
    if (g.G != g.Gc && g.mean_mode == 1) return false; // the cross-head forms take equal sizes only
    if (a.g > 8) return false;
    if (g.mean_mode == 1 && a.n_q_heads > 64) return false; // the dense mean terms keep all query heads of a sequence in LDS
    if (a.batch * a.n_kv_heads > 65535) return false;
    // the kernels address record fields with compile-time offsets
    DoMatch m;
    pick(a, m);
    return m.result;
}

int decode_mfma_splits(const DecodeArgs &a)
{
    if (!decode_mfma_supported(a)) return 1;
    DoPlan p;
    pick(a, p);
    return p.result;
}

void set_split_timing_events(hipEvent_t begin, hipEvent_t end)
{
    t_ev_begin = begin;
    t_ev_end = end;
}

hipError_t launch_decode_split_mfma(const DecodeArgs &a, hipStream_t s)
{
    if (!decode_mfma_supported(a)) return hipErrorInvalidValue;
    if (a.geom.mean_mode == 1 && !xhead_fused_fmt(a)) {
        if (!a.xs || !a.xp || !a.xmc) return hipErrorInvalidValue;
        const hipError_t e = launch_xhead_scores(a, s);
        if (e != hipSuccess) return e;
    }
    DoLaunch l;
    l.s = s;
    pick(a, l);
    return l.result;
}

} // namespace tadakv

#ifdef TADA_PHASE_CLOCK
// out[0..13]: cycles summed over all waves per phase; out[14]: loop iterations; out[15]: waves.
// reset != 0 clears the sums afterwards.
extern "C" int kv_debug_phase_clocks(unsigned long long *out, int reset)
{
    if (hipDeviceSynchronize() != hipSuccess) return -1;
    if (hipMemcpyFromSymbol(out, HIP_SYMBOL(tadakv::tada_phase_clk), 16 * sizeof(unsigned long long)) != hipSuccess) return -1;
    if (reset) {
        unsigned long long z[16] = {};
        if (hipMemcpyToSymbol(HIP_SYMBOL(tadakv::tada_phase_clk), z, sizeof(z)) != hipSuccess) return -1;
    }
    return 0;
}
#endif
