// Value projection fused with the compression of the values (gfx950): Algorithm 1 step 3 of
// arxiv 2506.04642, "CompressV(X, W_V)" (Sec. 3.4; App. A "Compressing value activations": the
// linear projection that produces the values is the only operator in front of their mean-centring
// and quantisation, so the two are one kernel and the projected values never travel through memory
// as a tensor of their own).
//
//   V[t][o] = sum_k X[t][k] * W_V[o][k]      16-bit operands, binary32 accumulation on the matrix
//                                            cores, the sum rounded (nearest even) to the 16-bit type
// followed, for every whole block of 32 tokens of one (sequence, kv head), by the value side of the
// quantiser (block mean per channel, deviation, one (scale, zero) per token and group of Gc
// channels, codes, packed words: quant_wave.h) on the accumulator tile, or, for tokens that stay
// in the raw residual buffer (Sec. 3.3), by a store of the rounded rows into that buffer.
//
// compressv_gemm_kernel: a workgroup owns 256 tokens (eight groups of 32) x NH kv heads (128
// channels each); wave (wm, wn) owns tokens 64 wm .. + 63 of head wn: 4 x 8 tiles of
// v_mfma_f32_16x16x32 accumulators, i.e. two quantiser items, two waves per SIMD.  X and W_V tiles
// of 64 k-values (rows of 128 bytes, whole cache lines) are fetched straight into LDS
// (global_load_lds_dwordx4) a stage ahead, 16-byte pieces of a row XOR-swizzled by the row so that
// the operand reads (16 rows x one piece) hit distinct banks.
// Every output element is one chain of model_dim / 32 matrix instructions in ascending k, the same
// chain in project_rows_kernel below, so a token's projected value does not depend on which of
// the two kernels, or which tile, produced it.
//
// project_rows_kernel: the decode step's shape (a handful of rows against the whole of W_V): one
// wave per 16 output channels and 16 rows, its operands streamed with sixteen steps in flight.
#include "quant_wave.h"

namespace tadakv {
namespace {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4))); // one matrix operand: eight 16-bit values
typedef const __attribute__((address_space(1))) void *gptr_t;
typedef __attribute__((address_space(3))) void *lptr_t;

constexpr int kTileTokens = 256; // tokens per workgroup
constexpr int kStepK = 64;       // k-values per stage: rows of 128 bytes, whole cache lines
constexpr int kEpiBytes = 16384; // per wave after the main loop: transposed 16-bit tile + record image
constexpr int kTTStride = 80;    // bytes per channel column of the transposed tile (32 tokens + pad)

template <int DT> __device__ __forceinline__ v4f mfma16(const u32x4 &a, const u32x4 &b, v4f c)
{
    if (DT == 1) return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(v8bf, a), __builtin_bit_cast(v8bf, b), c, 0, 0, 0);
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(v8h, a), __builtin_bit_cast(v8h, b), c, 0, 0, 0);
}
template <int DT> __device__ __forceinline__ v4f mfma16(const uint4 &a, const uint4 &b, v4f c)
{
    return mfma16<DT>(u32x4{a.x, a.y, a.z, a.w}, u32x4{b.x, b.y, b.z, b.w}, c);
}

// LDS operand read issued by hand.  The compiler makes every LDS read it knows of wait for all
// outstanding direct-to-LDS fetches (it cannot tell which buffer they fill), which would undo the
// fetch-ahead of the main loop; these reads are invisible to that rule.  The result must not be used
// before lds_reads_done has been given the same registers.
template <int OFF> __device__ __forceinline__ void lds_read16(u32x4 &dst, uint32_t addr)
{
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(OFF));
}
__device__ __forceinline__ void lds_reads_done(u32x4 (&a)[4], u32x4 (&b)[8])
{
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(b[0]), "+v"(b[1]), "+v"(b[2]), "+v"(b[3]),
                   "+v"(b[4]), "+v"(b[5]), "+v"(b[6]), "+v"(b[7]));
}

// two binary32 values rounded (nearest even) to the 16-bit type, packed low | high << 16
template <int DT> __device__ __forceinline__ uint32_t narrow2(float lo, float hi)
{
    if (DT == 1) {
        const __bf16 a = (__bf16)lo, b = (__bf16)hi;
        return (uint32_t) * (const uint16_t *)&a | ((uint32_t) * (const uint16_t *)&b << 16);
    }
    return (uint32_t)f16_rne(lo) | ((uint32_t)f16_rne(hi) << 16);
}
// the 16-bit pattern of a binary32 value that is exactly representable in the type
template <int DT> __device__ __forceinline__ uint32_t bits16_exact(float f)
{
    if (DT == 1) return __float_as_uint(f) >> 16;
    return (uint32_t)f16_rne(f);
}

// Group f of the launch: sequence (of the run), group inside the sequence, valid tokens.
struct GroupId {
    int b, gi, nv;
};
__device__ __forceinline__ GroupId group_of(const ProjectArgs &p, int f)
{
    GroupId g;
    g.b = f / p.n_groups;
    g.gi = f % p.n_groups;
    const int left = p.n_tok - 32 * g.gi;
    g.nv = left < 32 ? left : 32;
    return g;
}

// The rounded 32-token x 128-channel tile of one (group, kv head), held by a wave in the
// quantiser's lane layout x[token j][channel e] (tokens 8 tg + j, channels 8 c8 + e), goes where
// the launch says: into the record of block first_block + gi (values' part: codes, metadata,
// mean), or as raw rows into the residual buffer; and, if asked for, into the caller's tensor.
template <int DT, int GC, int BITS>
__device__ __forceinline__ void tile_out(const ProjectArgs &p, float (&x)[8][8], const GroupId &g, int h, int lane,
                                         unsigned char *img, uint32_t mean_pair)
{
    constexpr int G = 32, NGV = kHeadDim / GC;
    const LayerGeom &gm = p.geom;
    const int tg = lane & 3, c8 = lane >> 2;
    if (p.v_out || p.mode == 1) {
#pragma unroll
        for (int j = 0; j < 8; j++) {
            const int t = 8 * tg + j;
            uint4 row;
            row.x = bits16_exact<DT>(x[j][0]) | (bits16_exact<DT>(x[j][1]) << 16);
            row.y = bits16_exact<DT>(x[j][2]) | (bits16_exact<DT>(x[j][3]) << 16);
            row.z = bits16_exact<DT>(x[j][4]) | (bits16_exact<DT>(x[j][5]) << 16);
            row.w = bits16_exact<DT>(x[j][6]) | (bits16_exact<DT>(x[j][7]) << 16);
            if (t < g.nv) {
                const int tn = p.t0 + 32 * g.gi + t; // token of the call
                if (p.v_out)
                    *(uint4 *)(p.v_out + (long long)g.b * p.vo_stride_b + (long long)tn * p.vo_stride_t +
                               (long long)h * p.vo_stride_h + c8 * 8) = row;
                if (p.mode == 1) {
                    const long long u = (long long)(p.b0 + g.b) * p.n_kv_heads + h;
                    *(uint4 *)(p.layer + gm.v_resid_off + (u * gm.R + p.dst_row + 32 * g.gi + t) * (kHeadDim * 2) + c8 * 16) = row;
                }
            }
        }
    }
    if (p.mode == 1) return;

    // ---- the quantiser's value side on the tile (Eq. 1-4 with the per-channel block mean, or no mean)
    const int base_off = gm.v_codes;
    if (gm.mean_mode == 0) {
        // mean_pair: the binary16 means of channels 2 lane and 2 lane + 1 (the caller formed the sums over
        // the block's tokens, in token order, with a channel's 32 tokens in one lane); the record's mean
        // row is the lanes' words in order, and channels 8 c8 + 2 k and + 2 k + 1 are quad lane k's
        *(uint32_t *)(img + (gm.v_mean - base_off) + lane * 4) = mean_pair;
        const uint32_t q0 = quad_bcast_u<0>(mean_pair), q1 = quad_bcast_u<1>(mean_pair), q2 = quad_bcast_u<2>(mean_pair),
                       q3 = quad_bcast_u<3>(mean_pair);
        float m[8];
        m[0] = f16_val((uint16_t)(q0 & 0xFFFFu)); m[1] = f16_val((uint16_t)(q0 >> 16));
        m[2] = f16_val((uint16_t)(q1 & 0xFFFFu)); m[3] = f16_val((uint16_t)(q1 >> 16));
        m[4] = f16_val((uint16_t)(q2 & 0xFFFFu)); m[5] = f16_val((uint16_t)(q2 >> 16));
        m[6] = f16_val((uint16_t)(q3 & 0xFFFFu)); m[7] = f16_val((uint16_t)(q3 >> 16));
#pragma unroll
        for (int j = 0; j < 8; j++)
#pragma unroll
            for (int e = 0; e < 8; e++) x[j][e] = x[j][e] - m[e];
    } else {
#pragma unroll
        for (int j = 0; j < 8; j++)
#pragma unroll
            for (int e = 0; e < 8; e++) x[j][e] = x[j][e] - 0.0f;
    }
    emit_value_half<GC, BITS, 2>(x, 0, lane, img, img + (gm.v_meta - base_off));
    const int part_bytes = (gm.mean_mode == 0 ? gm.v_mean + 256 : gm.v_meta + G * NGV * 4) - base_off;
    unsigned char *rec = p.layer + record_offset(gm, p.n_kv_heads, p.b0 + g.b, h, p.first_block + g.gi);
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); // this wave's LDS writes have landed
    for (int off = lane * 16; off < part_bytes; off += 64 * 16) *(uint4 *)(rec + base_off + off) = *(const uint4 *)(img + off);
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); // the image is in registers before the next group overwrites it
}

template <int N> __device__ __forceinline__ void wait_vm()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

template <int DT, int NH, int GC, int BITS>
__global__ __launch_bounds__(256 * NH) void compressv_gemm_kernel(ProjectArgs p)
{
    constexpr int NW = 4 * NH;                      // waves: 4 token quarters x NH heads
    constexpr int A_BYTES = kTileTokens * 128;      // X tile of a stage: 64 k-values, rows of 128 bytes
    constexpr int B_BYTES = NH * kHeadDim * 128;    // W_V tile of a stage
    constexpr int STAGE = A_BYTES + B_BYTES;
    constexpr int PER = STAGE / 1024 / NW;          // fetch instructions (1 KiB each) per wave and stage
    static_assert(STAGE / 1024 % NW == 0, "the stage divides among the waves");
    static_assert(NW * kEpiBytes <= 2 * STAGE, "the epilogue fits the staging buffers");
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[]; // two stages

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int wm = wave & 3, wn = wave >> 2;
    // Workgroups are dealt to the eight dies in turn: the ones that share a token tile (the head
    // groups of that tile) get ids a multiple of eight apart, so they run on one die and find the
    // tile's rows of X in its cache.
    const int HG = p.n_kv_heads / NH;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int tile = (slot / HG) * 8 + xcd, hg = slot % HG;
    const int n_f = p.batch * p.n_groups;
    if (tile * 8 >= n_f) return; // (the grid is padded to whole rounds of eight tiles)

    // ---- where this lane's pieces of a stage come from: instruction q of the stage fills rows
    // 8 q .. 8 q + 7 (128 bytes each: whole cache lines), lane l the piece (l & 7) ^ (row & 7) of row 8 q + (l >> 3)
    const uint16_t *src[PER];
    {
        const int r8 = lane >> 3, pc = (lane & 7) ^ r8;
#pragma unroll
        for (int i = 0; i < PER; i++) {
            const int q = wave * PER + i;
            if (q < A_BYTES / 1024) {
                const int row = 8 * q + r8;
                int f = tile * 8 + (row >> 5);
                f = f < n_f ? f : n_f - 1; // past the end: any valid row, the result is not stored
                const GroupId g = group_of(p, f);
                int t = row & 31;
                t = t < g.nv ? t : g.nv - 1;
                src[i] = p.x + (long long)g.b * p.x_stride_b + (long long)(p.t0 + 32 * g.gi + t) * p.x_stride_t + pc * 8;
            } else {
                const int row = 8 * (q - A_BYTES / 1024) + r8; // output channel within the workgroup's heads
                src[i] = p.w + ((long long)hg * NH * kHeadDim + row) * p.model_dim + pc * 8;
            }
        }
    }
    const int stages = p.model_dim / kStepK;
    auto issue = [&](int sg) { // stage sg (k-values 64 sg .. + 63; the last stage again beyond it) into buffer sg % 2
        const int sk = sg < stages ? sg : stages - 1;
#pragma unroll
        for (int i = 0; i < PER; i++) {
            const int q = wave * PER + i;
            __builtin_amdgcn_global_load_lds((gptr_t)(src[i] + (long long)sk * kStepK), (lptr_t)(lds + (sg & 1) * STAGE + q * 1024), 16, 0, 0);
        }
    };

    v4f acc[4][8];
#pragma unroll
    for (int mt = 0; mt < 4; mt++)
#pragma unroll
        for (int nt = 0; nt < 8; nt++) acc[mt][nt] = v4f{0.0f, 0.0f, 0.0f, 0.0f};

    const int n = lane & 15, kg = lane >> 4;
    // this lane's operand piece inside a 16-row tile (2 KiB) for the low and the high 32 k-values of
    // a stage: row n, piece 4 half + kg, swizzled by the row
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lptr_t)lds;
    const uint32_t a_base = lds0 + wm * (64 * 128) + n * 128, b_base = lds0 + A_BYTES + wn * (kHeadDim * 128) + n * 128;
    const uint32_t sw_lo = (uint32_t)((kg ^ (n & 7)) << 4), sw_hi = (uint32_t)(((4 + kg) ^ (n & 7)) << 4);
    u32x4 fa[2][4], fb[2][8]; // operands of the current half step and of the next one
    auto read_frags = [&](int sg, uint32_t sw, u32x4(&a)[4], u32x4(&b)[8]) {
        const uint32_t so = (uint32_t)((sg & 1) * STAGE) + sw;
        lds_read16<0>(a[0], a_base + so);
        lds_read16<2048>(a[1], a_base + so);
        lds_read16<4096>(a[2], a_base + so);
        lds_read16<6144>(a[3], a_base + so);
        lds_read16<0>(b[0], b_base + so);
        lds_read16<2048>(b[1], b_base + so);
        lds_read16<4096>(b[2], b_base + so);
        lds_read16<6144>(b[3], b_base + so);
        lds_read16<8192>(b[4], b_base + so);
        lds_read16<10240>(b[5], b_base + so);
        lds_read16<12288>(b[6], b_base + so);
        lds_read16<14336>(b[7], b_base + so);
    };
    auto mfmas = [&](u32x4(&a)[4], u32x4(&b)[8]) {
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int mt = 0; mt < 4; mt++)
#pragma unroll
            for (int nt = 0; nt < 8; nt++) acc[mt][nt] = mfma16<DT>(a[mt], b[nt], acc[mt][nt]);
        __builtin_amdgcn_sched_barrier(0);
    };

    // A stage is consumed in two half steps of 32 k-values (32 matrix instructions per wave each);
    // the operands of a half step are read from LDS while the matrix instructions of the half step
    // before it run.  Once a wave holds the high half's operands it is done with the stage's buffer;
    // at the one barrier of a stage everybody is, and everybody's part of the next stage (fetched one
    // stage earlier) has landed; then the stage after the next is fetched into the freed buffer and
    // the next stage's low operands are read.  Past the last stage the fetch repeats the last one into
    // a buffer nobody reads any more and the operand read returns unused data, so that every stage is
    // the same straight line of code.
    issue(0);
    issue(1);
    wait_vm<PER>(); // stage 0 has landed
    __builtin_amdgcn_s_barrier();
    read_frags(0, sw_lo, fa[0], fb[0]);
    for (int sg = 0; sg < stages; sg++) {
        lds_reads_done(fa[0], fb[0]);
        read_frags(sg, sw_hi, fa[1], fb[1]);
        mfmas(fa[0], fb[0]);
        lds_reads_done(fa[1], fb[1]);
        wait_vm<0>();
        __builtin_amdgcn_s_barrier();
        issue(sg + 2);
        read_frags(sg + 1, sw_lo, fa[0], fb[0]);
        mfmas(fa[1], fb[1]);
    }
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    __syncthreads(); // the staging buffers are free: each wave takes 16 KiB of them for its epilogue
    unsigned char *tt = lds + wave * kEpiBytes;  // [128 channels][32 tokens] 16-bit, kTTStride bytes per channel
    unsigned char *img = tt + kHeadDim * kTTStride; // the values' part of a record
    const int tg = lane & 3, c8 = lane >> 2;
    const int h = hg * NH + wn;
#pragma unroll
    for (int blk = 0; blk < 2; blk++) {
        const int f = tile * 8 + 2 * wm + blk;
        if (f >= n_f) break;
        const GroupId g = group_of(p, f);
        // accumulators (lane: tokens 16 mt + 4 kg .. + 3 of channel 16 nt + n), rounded, into the
        // transposed tile: the four tokens are 8 contiguous bytes
#pragma unroll
        for (int m2 = 0; m2 < 2; m2++)
#pragma unroll
            for (int nt = 0; nt < 8; nt++) {
                const v4f c = acc[2 * blk + m2][nt];
                *(uint2 *)(tt + (16 * nt + n) * kTTStride + (16 * m2 + 4 * kg) * 2) = uint2{narrow2<DT>(c[0], c[1]), narrow2<DT>(c[2], c[3])};
            }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        // back in the quantiser's layout: tokens 8 tg .. + 7 of channel 8 c8 + e are 16 contiguous bytes
        float x[8][8];
#pragma unroll
        for (int e = 0; e < 8; e++) {
            const uint4 pcs = *(const uint4 *)(tt + (8 * c8 + e) * kTTStride + tg * 16);
            const uint32_t wv[4] = {pcs.x, pcs.y, pcs.z, pcs.w};
#pragma unroll
            for (int k = 0; k < 4; k++) {
                x[2 * k][e] = widen16((uint16_t)(wv[k] & 0xFFFFu), DT);
                x[2 * k + 1][e] = widen16((uint16_t)(wv[k] >> 16), DT);
            }
        }
        // the per-channel sums of the block mean, over the tokens in order: a channel's 32 tokens are
        // 64 contiguous bytes of the transposed tile, so lane l adds up channels 2 l and 2 l + 1 (every
        // lane adds; in the quantiser's layout three quarters of a quad's adds would be masked)
        uint32_t mean_pair = 0u;
        if (p.geom.mean_mode == 0 && p.mode != 1) {
            float sm[2];
#pragma unroll
            for (int c = 0; c < 2; c++) {
                const unsigned char *col = tt + (2 * lane + c) * kTTStride;
                float sacc = 0.0f;
#pragma unroll
                for (int q = 0; q < 4; q++) {
                    const uint4 pcs = *(const uint4 *)(col + 16 * q);
                    const uint32_t wv[4] = {pcs.x, pcs.y, pcs.z, pcs.w};
#pragma unroll
                    for (int k = 0; k < 4; k++) {
                        sacc = sacc + widen16((uint16_t)(wv[k] & 0xFFFFu), DT);
                        sacc = sacc + widen16((uint16_t)(wv[k] >> 16), DT);
                    }
                }
                sm[c] = sacc;
            }
            mean_pair = (uint32_t)f16_rne(sm[0] / 32.0f) | ((uint32_t)f16_rne(sm[1] / 32.0f) << 16);
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); // the tile is in registers before the next group overwrites it
        tile_out<DT, GC, BITS>(p, x, g, h, lane, img, mean_pair);
    }
}

// A few rows (a decode step: one token per sequence) against all of W_V.  One wave per (16 output
// channels, 16 rows): B operand = its 16 rows of W_V, 16 bytes per lane and matrix instruction
// (k-values 32 s + 8 (l >> 4) .. + 7 of channel l & 15); A operand = its rows of X.  Sixteen steps
// of loads are in flight per lane: each step's registers are loaded again as soon as its matrix
// instruction has consumed them.  Same accumulation chain as the tiled kernel.
// Row r of the launch is token t0 + r % n_tok of sequence r / n_tok (of the run).
template <int DT>
__global__ __launch_bounds__(64) void project_rows_kernel(ProjectArgs p)
{
    const int lane = threadIdx.x, n = lane & 15, kg = lane >> 4;
    const int o0 = blockIdx.x * 16, r0 = blockIdx.y * 16; // first output channel, first row of the wave
    const int rows = p.batch * p.n_tok;
    const uint16_t *wrow = p.w + (long long)(o0 + n) * p.model_dim + 8 * kg;
    int ra = r0 + n;
    ra = ra < rows ? ra : rows - 1;
    const uint16_t *xrow = p.x + (long long)(ra / p.n_tok) * p.x_stride_b + (long long)(p.t0 + ra % p.n_tok) * p.x_stride_t + 8 * kg;
    v4f acc = v4f{0.0f, 0.0f, 0.0f, 0.0f};
    constexpr int D = 16; // steps in flight
    const int steps = p.model_dim / 32;
    uint4 a[D], b[D];
#pragma unroll
    for (int i = 0; i < D; i++) {
        const int s = i < steps ? i : steps - 1;
        b[i] = *(const uint4 *)(wrow + 32 * s);
        a[i] = *(const uint4 *)(xrow + 32 * s);
    }
    for (int s0 = 0; s0 < steps; s0 += D) {
#pragma unroll
        for (int i = 0; i < D; i++) {
            if (s0 + i < steps) acc = mfma16<DT>(a[i], b[i], acc);
            const int s = s0 + i + D < steps ? s0 + i + D : steps - 1;
            b[i] = *(const uint4 *)(wrow + 32 * s);
            a[i] = *(const uint4 *)(xrow + 32 * s);
        }
    }
    // lane: rows r0 + 4 kg .. + 3 of channel o0 + n
    const int o = o0 + n, h = o / kHeadDim, c = o % kHeadDim;
#pragma unroll
    for (int j = 0; j < 4; j++) {
        const int r = r0 + 4 * kg + j;
        if (r >= rows) continue;
        const int bb = r / p.n_tok, t = r % p.n_tok;
        const uint16_t v = (uint16_t)(narrow2<DT>(acc[j], 0.0f) & 0xFFFFu);
        if (p.v_out)
            p.v_out[(long long)bb * p.vo_stride_b + (long long)(p.t0 + t) * p.vo_stride_t + (long long)h * p.vo_stride_h + c] = v;
        const long long u = (long long)(p.b0 + bb) * p.n_kv_heads + h;
        *(uint16_t *)(p.layer + p.geom.v_resid_off + (u * p.geom.R + p.dst_row + t) * (kHeadDim * 2) + c * 2) = v;
    }
}

template <int DT, int NH, int GC, int BITS> hipError_t launch_gemm(const ProjectArgs &p, hipStream_t s)
{
    constexpr size_t lds = 2 * (size_t)(kTileTokens * 128 + NH * kHeadDim * 128);
    static const bool ready = hipFuncSetAttribute((const void *)compressv_gemm_kernel<DT, NH, GC, BITS>,
                                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) == hipSuccess;
    if (!ready) return note_launch(hipErrorInvalidValue);
    const long long n_f = (long long)p.batch * p.n_groups;
    const long long tiles = (n_f + 7) / 8, rounds = (tiles + 7) / 8;
    const long long grid = rounds * 8 * (p.n_kv_heads / NH);
    if (grid > 0x7FFFFFFF) return note_launch(hipErrorInvalidValue);
    hipLaunchKernelGGL((compressv_gemm_kernel<DT, NH, GC, BITS>), dim3((unsigned)grid), dim3(256 * NH), lds, s, p);
    return note_launch(hipGetLastError());
}
template <int DT, int NH> hipError_t launch_gemm_fmt(const ProjectArgs &p, hipStream_t s)
{
    const int gc = p.geom.Gc, b = p.geom.v_bits;
#define TADAKV_CV(GCV) (b == 2 ? launch_gemm<DT, NH, GCV, 2>(p, s) : b == 4 ? launch_gemm<DT, NH, GCV, 4>(p, s) : launch_gemm<DT, NH, GCV, 8>(p, s))
    return gc == 32 ? TADAKV_CV(32) : gc == 64 ? TADAKV_CV(64) : TADAKV_CV(128);
#undef TADAKV_CV
}

template <int DT> hipError_t launch_rows(const ProjectArgs &p, hipStream_t s)
{
    const int rows = p.batch * p.n_tok;
    const dim3 grid(p.n_kv_heads * kHeadDim / 16, (rows + 15) / 16), block(64);
    hipLaunchKernelGGL((project_rows_kernel<DT>), grid, block, 0, s, p);
    return note_launch(hipGetLastError());
}

} // namespace

bool compressv_supported(const LayerGeom &g)
{
    return g.G == 32 && g.k_bits == g.v_bits && (g.v_bits == 2 || g.v_bits == 4 || g.v_bits == 8) && g.mean_mode != 1;
}

hipError_t launch_compressv(const ProjectArgs &p, hipStream_t s)
{
    if (!compressv_supported(p.geom) || p.model_dim % kStepK || p.n_groups < 1 || p.n_tok < 1 || p.batch < 1)
        return note_launch(hipErrorInvalidValue);
    (void)hipGetLastError(); // drop any stale error left by earlier runtime calls of this thread
    // raw rows of a decode step: the streaming kernel
    if (p.mode == 1 && (long long)p.batch * p.n_tok <= 256)
        return p.geom.dtype == 1 ? launch_rows<1>(p, s) : launch_rows<0>(p, s);
    if (p.n_kv_heads % 2 == 0) return p.geom.dtype == 1 ? launch_gemm_fmt<1, 2>(p, s) : launch_gemm_fmt<0, 2>(p, s);
    return p.geom.dtype == 1 ? launch_gemm_fmt<1, 1>(p, s) : launch_gemm_fmt<0, 1>(p, s);
}

} // namespace tadakv
