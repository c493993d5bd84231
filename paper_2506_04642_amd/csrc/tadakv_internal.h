// Internal declarations shared by the host-side ABI and the HIP kernels of libtadakv.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tadakv {

constexpr int kHeadDim = 128;
constexpr int kMaxGroupQ = 8;       // query heads per kv head the kernels are sized for
constexpr int kPartialStride = 132; // floats per (unit, q head, split): O[128], max, sum, pad
constexpr int kMaxSplits = 256;
constexpr int kMaxRaggedBatch = 256; // sequences whose lengths may differ from one another

// Geometry of one layer's buffer; byte offsets, -1 where a field is absent.
struct LayerGeom {
    int k_bits, v_bits;
    int G, Gc, R, NB;     // group_tokens, group_channels, resid_cap, blocks per sequence
    int mean_mode, dtype;
    long long rec_bytes;
    int k_codes, k_scale, k_zero, k_mean;
    int v_codes, v_meta, v_mean;
    long long xmean_off, k_resid_off, v_resid_off, layer_bytes;
    // paged placement: block slots shared through a device table [batch][table_stride] (null: dense)
    const int32_t *table;
    int table_stride, pool;
};

// Block slot of logical block blk of sequence b.  Entries outside the pool are clamped into it.
__device__ __forceinline__ long long block_slot(const LayerGeom &g, int b, int blk)
{
    if (!g.table) return (long long)b * g.NB + blk;
    int p = g.table[(long long)b * g.table_stride + blk];
    p = p < 0 ? 0 : (p >= g.pool ? g.pool - 1 : p);
    return p;
}
// Byte offset of the record of (sequence b, kv head h, block blk) in the layer buffer.
__device__ __forceinline__ long long record_offset(const LayerGeom &g, int n_kv_heads, int b, int h, int blk)
{
    if (!g.table) return ((long long)(b * n_kv_heads + h) * g.NB + blk) * g.rec_bytes;
    return (block_slot(g, b, blk) * n_kv_heads + h) * g.rec_bytes;
}
// Byte offset of the cross-head mean tile [G][128] binary16 of (sequence b, block blk, K | V).
__device__ __forceinline__ long long xmean_offset(const LayerGeom &g, int b, int blk, int which)
{
    return g.xmean_off + ((block_slot(g, b, blk) * 2 + which) * g.G * kHeadDim) * 2;
}

// Device-resident lengths of one layer (for decode steps replayed from a HIP graph, whose kernel
// arguments cannot follow a growing cache): ints st[p * 2B + 2b] = packed blocks and st[p * 2B + 2b + 1]
// = raw tokens of sequence b in state p (0 or 1), st[4B] = which state is the current one; B = batch.
// A step's first kernel writes the state after the step into the other slot, its last one makes that
// slot the current one.  Counts are clamped to the layer's capacity, so stale or foreign contents
// cannot take an access out of the layer's buffers.
constexpr int kDevLenPad = 4;
__host__ __device__ inline int dev_len_ints(int batch) { return 4 * batch + kDevLenPad; }
__device__ __forceinline__ void dev_len(const int *st, int batch, int b, int after, int nb_cap, int r_cap, int &nb, int &r)
{
    const int p = (st[4 * batch] & 1) ^ after;
    nb = st[p * 2 * batch + 2 * b];
    r = st[p * 2 * batch + 2 * b + 1];
    nb = nb < 0 ? 0 : (nb > nb_cap ? nb_cap : nb);
    r = r < 0 ? 0 : (r > r_cap ? r_cap : r);
}

struct AppendArgs {
    LayerGeom geom;
    unsigned char *layer;   // device base of the layer buffer
    const uint16_t *k_new;  // device
    const uint16_t *v_new;
    long long stride_b, stride_t, stride_h; // elements
    int n_kv_heads, batch; // batch: sequences of this launch (a run b0 .. b0 + batch - 1 of the cache's)
    int b0;             // first sequence of the run in the cache; the input pointers already point at it
    int r_old;          // residual tokens before the call
    int first_block;    // index of the first block this call writes
    int n_flush_blocks; // blocks to compress
    int copy_src, copy_dst, copy_n; // raw tail: input tokens [copy_src, copy_src+copy_n) -> residual[copy_dst..]
    // rotary embedding applied to the new keys on their way in (0: none, 1: pairs (i, i + 64),
    // 2: pairs (2i, 2i + 1)); tables [n_new][64] binary32, device
    int rope;
    const float *rope_cos, *rope_sin;
    // 0: keys and values; 1: keys only; 2: values only (the other side of the call is handled by
    // another kernel: the value projection fused with the compression, Alg. 1 step 3).  Only the
    // one-wavefront-per-item quantiser (blocks of 32 tokens, one width) and the raw copy take 1 or 2.
    int sides;
    // not null: a decode step on device-resident lengths (dev_len).  The quantiser's launch first
    // stores one token per sequence at the sequence's own position in the raw buffer and writes the
    // state after the step; then it compresses a sequence's raw buffer only if that token fills it
    // (r_old = R - 1: the last row from the caller), as block number "packed blocks" of the state before.
    int *len_dev;
};

// Value projection fused with the compression (Alg. 1 step 3): one launch covers, for each sequence
// of a run, n_groups groups of up to 32 consecutive tokens of the call's input.
struct ProjectArgs {
    LayerGeom geom;
    unsigned char *layer;    // device base of the layer buffer
    const uint16_t *x;       // layer input rows, [sequence of the run][token of the call][model_dim]
    long long x_stride_b, x_stride_t; // elements
    const uint16_t *w;       // value projection weights [n_kv_heads * 128][model_dim], one row per output channel
    int model_dim;
    int n_kv_heads, batch, b0; // sequences of this launch and the first one's index in the cache
    int t0;                  // token of the call's input that group 0 starts at
    int n_groups, n_tok;     // groups per sequence; tokens per sequence they cover (the last group may be short)
    int mode;                // 0: group gi is compressed into block first_block + gi; 1: raw rows into the
                             // residual buffer, token i of the launch at row dst_row + i
    int first_block, dst_row;
    uint16_t *v_out;         // if not null: the projected values as a tensor [sequence][token][kv head][128]
    long long vo_stride_b, vo_stride_t, vo_stride_h;
};

struct DecodeArgs {
    LayerGeom geom;
    const unsigned char *layer;
    const uint16_t *q;   // [batch][Hq][128]
    float *ws;           // partials [U][g][n_splits][kPartialStride]
    float *out;          // [batch][Hq][128]
    uint16_t *out16;     // the same in the cache's 16-bit type, if not null (then `out` is not written)
    int n_kv_heads, n_q_heads, batch, g;
    int n_blocks;        // packed blocks in the layer
    int r;               // residual tokens
    int n_splits;
    int blocks_per_split;
    // matrix-core kernel only: the newest residual token (index r - 1) is not in the cache yet;
    // the kernel takes it from these rows and stores it (null: every token is in the cache)
    const uint16_t *k_fresh, *v_fresh;
    long long fresh_stride_b, fresh_stride_h; // elements
    // cross-head mean on the matrix-core path: the dense mean terms go through three arrays in the
    // workspace (null otherwise).  xs [batch][Hq][tcap]: q . mean_K of every packed token;
    // xp [batch][Hq][tcap]: softmax weight of every packed token relative to its chunk's maximum;
    // xmc [batch][Hq][tcap / 64 + 1]: that maximum (exp2 domain) per 64-token chunk.
    float *xs, *xp, *xmc;
    int tcap;
    // xo [batch][Hq][n_xr][128]: the value mean plane's share of the output, per range of chunks,
    // relative to the head's largest split maximum; the merge adds the ranges up
    float *xo;
    int n_xr;
    // sequences of different lengths: n_blocks and r above are the maxima, the kernels take each
    // sequence's own counts from these (ragged == 0: every sequence has n_blocks and r)
    int ragged;
    // not null: the kernels take every sequence's counts from these device-resident lengths (the state
    // after the step's append, dev_len) instead; n_blocks and r only size the launch.  The merge makes
    // that state the current one.
    int *len_dev;
    uint16_t nb_seq[kMaxRaggedBatch], r_seq[kMaxRaggedBatch]; // 1 KiB of the kernel arguments
};

// packed blocks / raw tokens of sequence b
__host__ __device__ inline int seq_blocks(const DecodeArgs &a, int b)
{
#if defined(__HIP_DEVICE_COMPILE__)
    if (a.len_dev) {
        int nb, r;
        dev_len(a.len_dev, a.batch, b, 1, a.geom.NB, a.geom.R, nb, r);
        return nb;
    }
#endif
    return a.ragged ? a.nb_seq[b] : a.n_blocks;
}
__host__ __device__ inline int seq_resid(const DecodeArgs &a, int b)
{
#if defined(__HIP_DEVICE_COMPILE__)
    if (a.len_dev) {
        int nb, r;
        dev_len(a.len_dev, a.batch, b, 1, a.geom.NB, a.geom.R, nb, r);
        return r;
    }
#endif
    return a.ragged ? a.r_seq[b] : a.r;
}

// reconstruction of a layer's contents: lengths and geometry as for a decode launch
struct DequantArgs {
    DecodeArgs d;
    float *k_out, *v_out; // [batch][t_cap][n_kv_heads][128] binary32, either may be null
    int t_cap;
};

// records the outcome of a launch for kv_last_hip_error and passes it through
hipError_t note_launch(hipError_t e);

hipError_t launch_flush(const AppendArgs &a, hipStream_t s);
hipError_t launch_resid_copy(const AppendArgs &a, hipStream_t s);
bool step_store_supported(const LayerGeom &g); // formats the device-length decode step serves (launch_flush with len_dev)
bool compressv_supported(const LayerGeom &g); // formats the fused value projection serves
hipError_t launch_compressv(const ProjectArgs &p, hipStream_t s);
hipError_t launch_decode_split_valu(const DecodeArgs &a, hipStream_t s);
hipError_t launch_decode_split_mfma(const DecodeArgs &a, hipStream_t s);
// the calling thread's next matrix-core split launch records its begin and end into these (one-shot; null cancels)
void set_split_timing_events(hipEvent_t begin, hipEvent_t end);
bool decode_mfma_supported(const DecodeArgs &a);
bool xhead_fused(const DecodeArgs &a); // cross-head mean: both mean terms inside the matrix-core split kernel
int decode_mfma_splits(const DecodeArgs &a); // preferred split count of the matrix-core kernel
hipError_t launch_decode_merge(const DecodeArgs &a, hipStream_t s);
hipError_t launch_dequant(const DequantArgs &q, hipStream_t s);
// cross-head mean, matrix-core path: scores of the queries against the key mean plane (before the
// split kernel) and the value mean plane's contribution to the partial outputs (before the merge)
hipError_t launch_xhead_scores(const DecodeArgs &a, hipStream_t s);
hipError_t launch_xhead_values(const DecodeArgs &a, hipStream_t s);
int xhead_values_resident(int n_q_heads);
// read-only streaming pass over a buffer (the benchmark's measured bandwidth ceiling)
hipError_t launch_stream_read(const void *buf, size_t bytes, unsigned long long *sink, hipStream_t s); // workgroups of the value-mean kernel the device holds at once

} // namespace tadakv
