// Host side of libtadakv: argument validation, layer geometry, length bookkeeping (the residual
// policy of Sec. 3.3 of arxiv 2506.04642) and dispatch of the HIP kernels.  No device memory is
// allocated here and nothing synchronises.
#include "../../include/tadakv.h"
#include "tadakv_internal.h"

#include <mutex>
#include <new>
#include <vector>

using namespace tadakv;

struct kv_cache {
    kv_config cfg;
    std::vector<uint8_t> k_bits, v_bits;
    std::vector<unsigned char *> layers;
    std::vector<LayerGeom> geom;
    std::vector<int> packed, resid; // tokens, [layer][sequence]
    int &P(int layer, int b) { return packed[(size_t)layer * cfg.batch + b]; }
    int &R(int layer, int b) { return resid[(size_t)layer * cfg.batch + b]; }
    int P(int layer, int b) const { return packed[(size_t)layer * cfg.batch + b]; }
    int R(int layer, int b) const { return resid[(size_t)layer * cfg.batch + b]; }
    bool uniform(int layer) const
    {
        for (int b = 1; b < cfg.batch; b++)
            if (P(layer, b) != P(layer, 0) || R(layer, b) != R(layer, 0)) return false;
        return true;
    }
    std::vector<uint8_t> active;    // batch-wide calls act on these sequences only (empty: on all)
    bool on(int b) const { return active.empty() || active[b] != 0; }
    const int32_t *table = nullptr; // paged placement: the caller's block table (device)
    int table_stride = 0;
    int decode_path = 0;
    int forced_splits = 0;
    size_t xhead_off = 0, xhead_bytes = 0; // cross-head mean: where its arrays start in the workspace, total size
    size_t xhead_xo_rel = 0;               // start of the value-mean output slots relative to xhead_off
    int *len_dev = nullptr;                // device-resident lengths (kv_cache_lengths_to_device), [layer][dev_len_ints]
    std::vector<int> len_image;            // what was last sent there (the copy's source stays alive)
};

namespace {

long long align_up(long long n, long long a) { return (n + a - 1) / a * a; }

bool bits_ok(int b) { return b == 2 || b == 4 || b == 8 || b == 16; }

kv_status check_config(const kv_config *c)
{
    if (!c) return KV_E_NULL;
    if (!c->k_bits || !c->v_bits) return KV_E_NULL;
    if (c->n_layers <= 0 || c->batch <= 0 || c->n_kv_heads <= 0 || c->n_q_heads <= 0) return KV_E_BAD_CONFIG;
    if (c->head_dim != kHeadDim) return KV_E_BAD_CONFIG;
    if (c->n_q_heads % c->n_kv_heads) return KV_E_BAD_CONFIG;
    if (c->n_q_heads / c->n_kv_heads > kMaxGroupQ) return KV_E_BAD_CONFIG;
    if (!(c->group_tokens == 32 || c->group_tokens == 64 || c->group_tokens == 128)) return KV_E_BAD_CONFIG;
    if (!(c->group_channels == 32 || c->group_channels == 64 || c->group_channels == 128)) return KV_E_BAD_CONFIG;
    if (c->max_tokens <= 0 || c->max_tokens % c->group_tokens) return KV_E_BAD_CONFIG;
    if (c->pool_blocks < 0) return KV_E_BAD_CONFIG;
    if (c->resid_cap <= 0 || c->resid_cap % c->group_tokens || c->resid_cap > c->max_tokens) return KV_E_BAD_CONFIG;
    if (!(c->dtype == KV_F16 || c->dtype == KV_BF16)) return KV_E_BAD_CONFIG;
    if (!(c->mean_mode == KV_MEAN_CHANNEL_BLOCK || c->mean_mode == KV_MEAN_CROSS_HEAD ||
          c->mean_mode == KV_MEAN_NONE))
        return KV_E_BAD_CONFIG;
    for (int l = 0; l < c->n_layers; l++)
        if (!bits_ok(c->k_bits[l]) || !bits_ok(c->v_bits[l])) return KV_E_BAD_BITS;
    for (int l = 0; l < c->n_layers; l++) // one raw side next to one packed side: no kernel yet
        if ((c->k_bits[l] == 16) != (c->v_bits[l] == 16)) return KV_E_UNSUPPORTED;
    if ((long long)c->batch * c->n_kv_heads > 65535) return KV_E_UNSUPPORTED; // units index a launch grid's second dimension
    return KV_OK;
}

// The storage format of one layer (documented in tadakv.h next to kv_layer_layout).
LayerGeom make_geom(const kv_config &c, int layer)
{
    LayerGeom g{};
    const int d = c.head_dim, G = c.group_tokens, Gc = c.group_channels;
    g.k_bits = c.k_bits[layer];
    g.v_bits = c.v_bits[layer];
    g.G = G;
    g.Gc = Gc;
    g.R = c.resid_cap;
    g.NB = c.max_tokens / G;
    g.mean_mode = c.mean_mode;
    g.dtype = c.dtype;
    const bool cm = c.mean_mode == KV_MEAN_CHANNEL_BLOCK;
    int off = 0;
    g.k_scale = g.k_zero = g.k_mean = g.v_meta = g.v_mean = -1;
    g.k_codes = off;
    off += G * d * g.k_bits / 8;
    if (g.k_bits != 16) {
        g.k_scale = off; off += d * 2;
        g.k_zero = off;  off += d * 2;
        if (cm) { g.k_mean = off; off += d * 2; }
    }
    g.v_codes = off;
    off += G * d * g.v_bits / 8;
    if (g.v_bits != 16) {
        g.v_meta = off; off += G * (d / Gc) * 4;
        if (cm) { g.v_mean = off; off += d * 2; }
    }
    g.rec_bytes = align_up(off, 256);
    const long long U = (long long)c.batch * c.n_kv_heads;
    // block slots: every sequence its own (dense), or a shared pool (paged)
    const long long slots = c.pool_blocks > 0 ? c.pool_blocks : (long long)c.batch * g.NB;
    g.pool = c.pool_blocks;
    long long total = align_up(slots * c.n_kv_heads * g.rec_bytes, 256);
    g.xmean_off = total;
    if (c.mean_mode == KV_MEAN_CROSS_HEAD)
        total = align_up(total + slots * 2 * G * d * 2, 256);
    g.k_resid_off = total;
    total = align_up(total + U * c.resid_cap * d * 2, 256);
    g.v_resid_off = total;
    total = align_up(total + U * c.resid_cap * d * 2, 256);
    g.layer_bytes = total;
    return g;
}

// Sequence splits for a layer holding n_blocks packed blocks and r raw tokens: enough
// workgroups to cover the 256 compute units several times over, but never fewer than a handful
// of blocks per split so that the per-split prologue and the merge stay small.
void choose_splits(const kv_config &c, int n_blocks, int r, int *n_splits, int *blocks_per_split)
{
    const long long U = (long long)c.batch * c.n_kv_heads;
    const int units_of_work = n_blocks + (r > 0 ? 1 : 0);
    const int min_blocks = (c.group_tokens >= 64) ? 4 : 8; // >= 256 tokens per split
    long long want = (2048 + U - 1) / U;                    // ~8 workgroups per compute unit
    long long cap = (units_of_work + min_blocks - 1) / min_blocks;
    long long ns = want < cap ? want : cap;
    if (ns < 1) ns = 1;
    if (ns > kMaxSplits) ns = kMaxSplits;
    int bps = (int)((units_of_work + ns - 1) / ns);
    if (bps < 1) bps = 1;
    ns = (units_of_work + bps - 1) / bps; // no empty split
    if (ns < 1) ns = 1;
    *n_splits = (int)ns;
    *blocks_per_split = bps;
}

// Upper bound of the matrix-core kernel's split count: it never launches more workgroups than
// fit on the device at once (at most 8 per compute unit on 256 units).
int mfma_split_bound(const kv_config &c)
{
    const long long U = (long long)c.batch * c.n_kv_heads;
    long long b = 2048 / U;
    if (b < 1) b = 1;
    if (b > kMaxSplits) b = kMaxSplits;
    return (int)b;
}

size_t workspace_need(const kv_config &c, int n_splits)
{
    return (size_t)c.batch * c.n_q_heads * n_splits * kPartialStride * sizeof(float);
}

// Largest split count any length of this configuration can ask for.
int worst_splits(const kv_config &c)
{
    int worst = 1;
    const int NB = c.max_tokens / c.group_tokens;
    for (int nb = 0; nb <= NB; nb++) {
        int ns, bps;
        choose_splits(c, nb, 1, &ns, &bps);
        if (ns > worst) worst = ns;
    }
    if (mfma_split_bound(c) > worst) worst = mfma_split_bound(c);
    return worst;
}

// Cross-head mean on the matrix-core path: behind the partials (sized for the largest split count)
// the workspace holds xs and xp, [batch][Hq][max_tokens] floats each, xmc,
// [batch][Hq][max_tokens / 64 + 1] floats, and xo, [batch][Hq][ranges][128] floats.
// Token ranges of the value-mean product: one resident round of workgroups per launch (three per
// compute unit on 256 units), at least four chunks each.
int xhead_range_cap(const kv_config &c)
{
    int r = 768 / c.batch;
    return r < 1 ? 1 : (r > 256 ? 256 : r);
}
int xhead_ranges(const kv_config &c, int n_blocks)
{
    const int chunks = (int)(((long long)n_blocks * c.group_tokens + 63) / 64);
    int r = chunks / 4;
    if (r > xhead_range_cap(c)) r = xhead_range_cap(c);
    return r < 1 ? 1 : r;
}
size_t xhead_offset(const kv_config &c) { return (size_t)align_up((long long)workspace_need(c, worst_splits(c)), 256); }
size_t xhead_xo_offset(const kv_config &c)
{
    const size_t rows = (size_t)c.batch * c.n_q_heads;
    return (size_t)align_up((long long)(xhead_offset(c) + rows * ((size_t)2 * c.max_tokens + c.max_tokens / 64 + 1) * sizeof(float)), 256);
}
size_t xhead_total(const kv_config &c)
{
    const size_t rows = (size_t)c.batch * c.n_q_heads;
    return xhead_xo_offset(c) + rows * xhead_range_cap(c) * kHeadDim * sizeof(float);
}

kv_status layer_ok(const kv_cache *k, int layer)
{
    if (!k) return KV_E_NULL;
    if (layer < 0 || layer >= k->cfg.n_layers) return KV_E_BAD_LAYER;
    return KV_OK;
}

kv_status fill_decode(const kv_cache *k, int layer, DecodeArgs *a)
{
    const kv_config &c = k->cfg;
    a->geom = k->geom[layer];
    if (c.pool_blocks > 0) {
        if (!k->table) return KV_E_BAD_CONFIG; // paged placement without a block table
        a->geom.table = k->table;
        a->geom.table_stride = k->table_stride;
    }
    a->layer = k->layers[layer];
    a->n_kv_heads = c.n_kv_heads;
    a->n_q_heads = c.n_q_heads;
    a->batch = c.batch;
    a->g = c.n_q_heads / c.n_kv_heads;
    a->tcap = c.max_tokens;
    // sequences may differ in length: the launch is planned for the longest, the kernels take
    // each sequence's own counts from the table
    // a sequence that is not active counts as empty for this launch (its output rows are zeros)
    a->ragged = 0;
    for (int b = 0; b < c.batch; b++) {
        if (!k->on(b) && (k->P(layer, b) || k->R(layer, b))) a->ragged = 1;
        if (k->on(b) != k->on(0) || k->P(layer, b) != k->P(layer, 0) || k->R(layer, b) != k->R(layer, 0)) a->ragged = 1;
    }
    if (a->ragged && c.batch > kMaxRaggedBatch) return KV_E_UNSUPPORTED;
    a->n_blocks = 0;
    a->r = 0;
    for (int b = 0; b < c.batch; b++) {
        const int nb = k->on(b) ? k->P(layer, b) / c.group_tokens : 0, r = k->on(b) ? k->R(layer, b) : 0;
        if (nb > a->n_blocks) a->n_blocks = nb;
        if (r > a->r) a->r = r;
        if (a->ragged) {
            if (nb > 65535 || r > 65535) return KV_E_UNSUPPORTED; // the table holds 16-bit counts
            a->nb_seq[b] = (uint16_t)nb;
            a->r_seq[b] = (uint16_t)r;
        }
    }
    if (a->n_blocks == 0 && a->r == 0) return KV_E_EMPTY;
    choose_splits(c, a->n_blocks, a->r, &a->n_splits, &a->blocks_per_split);
    if (k->decode_path != 1 && decode_mfma_supported(*a)) {
        // the matrix-core kernel interleaves its splits chunk by chunk and sizes the launch to
        // the device; blocks_per_split is not used by it
        a->n_splits = decode_mfma_splits(*a);
        const int cap = mfma_split_bound(c);
        if (a->n_splits > cap) a->n_splits = cap;
    }
    if (k->forced_splits > 0) {
        const int work = a->n_blocks + (a->r > 0 ? 1 : 0);
        int ns = k->forced_splits < work ? k->forced_splits : work;
        a->blocks_per_split = (work + ns - 1) / ns;
        a->n_splits = (work + a->blocks_per_split - 1) / a->blocks_per_split;
    }
    return KV_OK;
}

bool use_mfma(const kv_cache *k, const DecodeArgs &a)
{
    if (k->decode_path == 1) return false;
    return decode_mfma_supported(a);
}

// Start of the cross-head arrays in the workspace: behind the partials of the largest automatic
// split count, or of this launch's own count where a forced count exceeds that.
size_t xhead_start(const kv_cache *k, const DecodeArgs &a)
{
    const size_t own = (size_t)align_up((long long)workspace_need(k->cfg, a.n_splits), 256);
    return own > k->xhead_off ? own : k->xhead_off;
}

// Workspace bytes this launch needs (the cross-head arrays included where the launch uses them).
size_t launch_workspace_need(const kv_cache *k, const DecodeArgs &a)
{
    const kv_config &c = k->cfg;
    const bool xhead = c.mean_mode == KV_MEAN_CROSS_HEAD && a.geom.k_bits != 16 && use_mfma(k, a) && !xhead_fused(a);
    return xhead ? xhead_start(k, a) + (k->xhead_bytes - k->xhead_off) : workspace_need(c, a.n_splits);
}

// Checks the workspace against this launch's need and places the cross-head arrays in it.
kv_status bind_workspace(const kv_cache *k, DecodeArgs *a, void *workspace, size_t workspace_bytes)
{
    const kv_config &c = k->cfg;
    // cross-head mean on the matrix-core path: the dense mean terms go through the workspace unless the
    // layer's format has the form of the split kernel that takes them in
    const bool xhead = c.mean_mode == KV_MEAN_CROSS_HEAD && a->geom.k_bits != 16 && use_mfma(k, *a) && !xhead_fused(*a);
    if (!workspace || workspace_bytes < launch_workspace_need(k, *a)) return KV_E_WORKSPACE;
    if ((uintptr_t)workspace % 256) return KV_E_ALIGN;
    a->ws = (float *)workspace;
    if (xhead) {
        const size_t rows = (size_t)c.batch * c.n_q_heads;
        const size_t start = xhead_start(k, *a);
        a->xs = (float *)((unsigned char *)workspace + start);
        a->xp = a->xs + rows * c.max_tokens;
        a->xmc = a->xp + rows * c.max_tokens;
        a->xo = (float *)((unsigned char *)workspace + start + k->xhead_xo_rel);
        a->n_xr = xhead_ranges(c, a->n_blocks);
        // one resident round of workgroups, whatever the compiler made of the kernel's registers
        const int fit = xhead_values_resident(c.n_q_heads) / c.batch;
        if (fit >= 1 && a->n_xr > fit) a->n_xr = fit;
    }
    return KV_OK;
}

} // namespace

namespace tadakv {
static thread_local hipError_t g_last_hip = hipSuccess;
hipError_t note_launch(hipError_t e)
{
    if (e != hipSuccess) g_last_hip = e;
    return e;
}
} // namespace tadakv

extern "C" {

const char *kv_last_hip_error(void) { return hipGetErrorString(tadakv::g_last_hip); }

const char *kv_strerror(kv_status s)
{
    switch (s) {
    case KV_OK: return "ok";
    case KV_E_NULL: return "null pointer";
    case KV_E_BAD_CONFIG: return "unsupported configuration";
    case KV_E_BAD_BITS: return "bit width must be 2, 4, 8 or 16";
    case KV_E_BAD_LAYER: return "layer index out of range";
    case KV_E_CAPACITY: return "append exceeds max_tokens";
    case KV_E_WORKSPACE: return "workspace missing or too small";
    case KV_E_ALIGN: return "misaligned pointer or stride";
    case KV_E_HIP: return "kernel launch failed";
    case KV_E_EMPTY: return "cache holds no token";
    case KV_E_UNSUPPORTED: return "configuration has no GPU path yet";
    }
    return "unknown status";
}

kv_status kv_cache_bytes(const kv_config *cfg, int32_t layer, size_t *bytes)
{
    if (!bytes) return KV_E_NULL;
    kv_status st = check_config(cfg);
    if (st != KV_OK) return st;
    if (layer < 0 || layer >= cfg->n_layers) return KV_E_BAD_LAYER;
    *bytes = (size_t)make_geom(*cfg, layer).layer_bytes;
    return KV_OK;
}

kv_status kv_workspace_bytes(const kv_config *cfg, size_t *bytes)
{
    if (!bytes) return KV_E_NULL;
    kv_status st = check_config(cfg);
    if (st != KV_OK) return st;
    // the split count grows with the length: sized for the largest over all reachable lengths
    *bytes = cfg->mean_mode == KV_MEAN_CROSS_HEAD ? xhead_total(*cfg) : workspace_need(*cfg, worst_splits(*cfg));
    return KV_OK;
}

kv_status kv_cache_create(const kv_config *cfg, void *const *layer_dev_ptrs, kv_cache **out)
{
    if (!out || !layer_dev_ptrs) return KV_E_NULL;
    kv_status st = check_config(cfg);
    if (st != KV_OK) return st;
    for (int l = 0; l < cfg->n_layers; l++) {
        if (!layer_dev_ptrs[l]) return KV_E_NULL;
        if ((uintptr_t)layer_dev_ptrs[l] % 256) return KV_E_ALIGN;
    }
    kv_cache *k = new (std::nothrow) kv_cache();
    if (!k) return KV_E_BAD_CONFIG;
    k->cfg = *cfg;
    k->k_bits.assign(cfg->k_bits, cfg->k_bits + cfg->n_layers);
    k->v_bits.assign(cfg->v_bits, cfg->v_bits + cfg->n_layers);
    k->cfg.k_bits = k->k_bits.data();
    k->cfg.v_bits = k->v_bits.data();
    for (int l = 0; l < cfg->n_layers; l++) {
        k->layers.push_back((unsigned char *)layer_dev_ptrs[l]);
        k->geom.push_back(make_geom(k->cfg, l));
    }
    k->packed.assign((size_t)cfg->n_layers * cfg->batch, 0);
    k->resid.assign((size_t)cfg->n_layers * cfg->batch, 0);
    if (cfg->mean_mode == KV_MEAN_CROSS_HEAD) {
        k->xhead_off = xhead_offset(k->cfg);
        k->xhead_bytes = xhead_total(k->cfg);
        k->xhead_xo_rel = xhead_xo_offset(k->cfg) - k->xhead_off;
    }
    *out = k;
    return KV_OK;
}

kv_status kv_cache_set_active(kv_cache *cache, const uint8_t *active, int32_t n)
{
    if (!cache) return KV_E_NULL;
    if (!active) {
        cache->active.clear();
        return KV_OK;
    }
    if (n != cache->cfg.batch) return KV_E_BAD_CONFIG;
    cache->active.assign(active, active + n);
    return KV_OK;
}

kv_status kv_cache_set_block_table(kv_cache *cache, const int32_t *table_dev, int32_t stride)
{
    if (!cache) return KV_E_NULL;
    const kv_config &c = cache->cfg;
    if (c.pool_blocks <= 0) return KV_E_BAD_CONFIG;
    if (!table_dev) return KV_E_NULL;
    if ((uintptr_t)table_dev % 4) return KV_E_ALIGN;
    if (stride < c.max_tokens / c.group_tokens) return KV_E_BAD_CONFIG;
    cache->table = table_dev;
    cache->table_stride = stride;
    return KV_OK;
}

kv_status kv_cache_destroy(kv_cache *cache)
{
    if (!cache) return KV_E_NULL;
    delete cache;
    return KV_OK;
}

kv_status kv_cache_reset(kv_cache *cache, int32_t layer)
{
    if (!cache) return KV_E_NULL;
    if (layer >= cache->cfg.n_layers) return KV_E_BAD_LAYER;
    for (int l = 0; l < cache->cfg.n_layers; l++)
        if (layer < 0 || l == layer)
            for (int b = 0; b < cache->cfg.batch; b++) cache->P(l, b) = cache->R(l, b) = 0;
    return KV_OK;
}

kv_status kv_cache_reset_seq(kv_cache *cache, int32_t layer, int32_t seq)
{
    if (!cache) return KV_E_NULL;
    if (layer >= cache->cfg.n_layers) return KV_E_BAD_LAYER;
    if (seq < 0 || seq >= cache->cfg.batch) return KV_E_BAD_CONFIG;
    for (int l = 0; l < cache->cfg.n_layers; l++)
        if (layer < 0 || l == layer) cache->P(l, seq) = cache->R(l, seq) = 0;
    return KV_OK;
}

kv_status kv_cache_len_seq(const kv_cache *cache, int32_t layer, int32_t seq, int32_t *packed, int32_t *resid)
{
    kv_status st = layer_ok(cache, layer);
    if (st != KV_OK) return st;
    if (!packed || !resid) return KV_E_NULL;
    if (seq < 0 || seq >= cache->cfg.batch) return KV_E_BAD_CONFIG;
    *packed = cache->P(layer, seq);
    *resid = cache->R(layer, seq);
    return KV_OK;
}

kv_status kv_cache_len(const kv_cache *cache, int32_t layer, int32_t *packed, int32_t *resid)
{
    kv_status st = layer_ok(cache, layer);
    if (st != KV_OK) return st;
    if (!packed || !resid) return KV_E_NULL;
    if (!cache->uniform(layer)) return KV_E_UNSUPPORTED; // the sequences differ: ask per sequence
    *packed = cache->P(layer, 0);
    *resid = cache->R(layer, 0);
    return KV_OK;
}

kv_status kv_cache_describe(const kv_cache *cache, int32_t layer, kv_layer_layout *out)
{
    kv_status st = layer_ok(cache, layer);
    if (st != KV_OK) return st;
    if (!out) return KV_E_NULL;
    const LayerGeom &g = cache->geom[layer];
    out->k_bits = g.k_bits;
    out->v_bits = g.v_bits;
    out->rec_bytes = g.rec_bytes;
    out->k_codes = g.k_codes;
    out->k_scale = g.k_scale;
    out->k_zero = g.k_zero;
    out->k_mean = g.k_mean;
    out->v_codes = g.v_codes;
    out->v_meta = g.v_meta;
    out->v_mean = g.v_mean;
    out->xmean_off = g.xmean_off;
    out->k_resid_off = g.k_resid_off;
    out->v_resid_off = g.v_resid_off;
    out->layer_bytes = g.layer_bytes;
    return KV_OK;
}

// rope: 0 none, 1 pairs (i, i + d/2), 2 pairs (2i, 2i + 1)
// Sequences seq0 .. seq0 + n_seq - 1 of the cache each take n_new tokens; input row (b, t, h) of
// the run is at b*stride_b + t*stride_t + h*stride_h from k_new / v_new.  Runs of sequences that
// hold the same number of tokens go into one launch.
// masked: a batch-wide call, which leaves out the sequences that are not active
static kv_status append_impl(kv_cache *cache, int32_t layer, int seq0, int n_seq, bool masked, const void *k_new, const void *v_new,
                             int32_t n_new, int64_t stride_b, int64_t stride_t, int64_t stride_h,
                             int rope, const float *rope_cos, const float *rope_sin, void *stream)
{
    kv_status st = layer_ok(cache, layer);
    if (st != KV_OK) return st;
    if (n_new < 0) return KV_E_BAD_CONFIG;
    if (n_new == 0) return KV_OK;
    if (!k_new || !v_new) return KV_E_NULL;
    const kv_config &c = cache->cfg;
    if (((uintptr_t)k_new % 16) || ((uintptr_t)v_new % 16)) return KV_E_ALIGN;
    if (stride_b % 8 || stride_t % 8 || stride_h % 8) return KV_E_ALIGN;
    if (stride_h < c.head_dim || stride_t < 0 || stride_b < 0) return KV_E_BAD_CONFIG;
    if (rope != 0) {
        if (!rope_cos || !rope_sin) return KV_E_NULL;
        if (((uintptr_t)rope_cos % 16) || ((uintptr_t)rope_sin % 16)) return KV_E_ALIGN;
    }
    if (c.pool_blocks > 0 && !cache->table) return KV_E_BAD_CONFIG; // paged placement without a block table
    auto takes = [&](int b) { return !masked || cache->on(b); };
    for (int b = seq0; b < seq0 + n_seq; b++)
        if (takes(b) && (long long)cache->P(layer, b) + cache->R(layer, b) + n_new > c.max_tokens) return KV_E_CAPACITY;
    const int G = c.group_tokens, R = c.resid_cap;
    // every limit of the launches below is checked here, before the first of them: an error leaves
    // nothing enqueued (the kernels number their work items, two per block and unit, with an int)
    if (((long long)R + n_new) / G * n_seq * c.n_kv_heads * 2 > 0x7FFFFFFFLL) return KV_E_UNSUPPORTED;
    hipStream_t s = (hipStream_t)stream;
    for (int b0 = seq0; b0 < seq0 + n_seq;) {
        if (!takes(b0)) {
            b0++;
            continue;
        }
        int b1 = b0 + 1;
        while (b1 < seq0 + n_seq && takes(b1) && cache->P(layer, b1) == cache->P(layer, b0) && cache->R(layer, b1) == cache->R(layer, b0)) b1++;
        const int r_old = cache->R(layer, b0);
        const long long total = (long long)r_old + n_new;
        const long long n_flush_tok = total / R * R;
        AppendArgs a{};
        a.geom = cache->geom[layer];
        a.geom.table = cache->table;
        a.geom.table_stride = cache->table_stride;
        a.layer = cache->layers[layer];
        a.k_new = (const uint16_t *)k_new + (long long)(b0 - seq0) * stride_b;
        a.v_new = (const uint16_t *)v_new + (long long)(b0 - seq0) * stride_b;
        a.stride_b = stride_b;
        a.stride_t = stride_t;
        a.stride_h = stride_h;
        a.n_kv_heads = c.n_kv_heads;
        a.batch = b1 - b0;
        a.b0 = b0;
        a.r_old = r_old;
        a.first_block = cache->P(layer, b0) / G;
        a.rope = rope;
        a.rope_cos = rope_cos;
        a.rope_sin = rope_sin;
        a.n_flush_blocks = (int)(n_flush_tok / G);
        if (n_flush_tok > 0) {
            a.copy_src = (int)(n_flush_tok - r_old);
            a.copy_dst = 0;
            a.copy_n = (int)(total - n_flush_tok);
        } else {
            a.copy_src = 0;
            a.copy_dst = r_old;
            a.copy_n = n_new;
        }
        if (a.n_flush_blocks > 0 && launch_flush(a, s) != hipSuccess) return KV_E_HIP;
        if (a.copy_n > 0 && launch_resid_copy(a, s) != hipSuccess) return KV_E_HIP;
        for (int b = b0; b < b1; b++) {
            cache->P(layer, b) += (int)n_flush_tok;
            cache->R(layer, b) = (int)(total - n_flush_tok);
        }
        b0 = b1;
    }
    return KV_OK;
}

kv_status kv_quant_append(kv_cache *cache, int32_t layer, const void *k_new, const void *v_new,
                          int32_t n_new, int64_t stride_b, int64_t stride_t, int64_t stride_h,
                          void *stream)
{
    if (!cache) return KV_E_NULL;
    return append_impl(cache, layer, 0, cache->cfg.batch, true, k_new, v_new, n_new, stride_b, stride_t, stride_h, 0, nullptr,
                       nullptr, stream);
}

kv_status kv_quant_append_seq(kv_cache *cache, int32_t layer, int32_t seq, const void *k_new, const void *v_new,
                              int32_t n_new, int64_t stride_t, int64_t stride_h, void *stream)
{
    if (!cache) return KV_E_NULL;
    if (seq < 0 || seq >= cache->cfg.batch) return KV_E_BAD_CONFIG;
    return append_impl(cache, layer, seq, 1, false, k_new, v_new, n_new, 0, stride_t, stride_h, 0, nullptr, nullptr, stream);
}

kv_status kv_rope_quant_append(kv_cache *cache, int32_t layer, const void *k_pre, const void *v_new,
                               int32_t n_new, int64_t stride_b, int64_t stride_t, int64_t stride_h,
                               const float *rope_cos, const float *rope_sin, int32_t pairing, void *stream)
{
    if (!cache) return KV_E_NULL;
    if (pairing != KV_ROPE_HALF && pairing != KV_ROPE_INTERLEAVED) return KV_E_BAD_CONFIG;
    return append_impl(cache, layer, 0, cache->cfg.batch, true, k_pre, v_new, n_new, stride_b, stride_t, stride_h,
                       pairing == KV_ROPE_HALF ? 1 : 2, rope_cos, rope_sin, stream);
}

kv_status kv_compressv_append(kv_cache *cache, int32_t layer, const void *k_new, int64_t k_stride_b, int64_t k_stride_t,
                              int64_t k_stride_h, const void *x, int64_t x_stride_b, int64_t x_stride_t, const void *w_v,
                              int32_t model_dim, int32_t n_new, const float *rope_cos, const float *rope_sin,
                              int32_t pairing, void *v_proj, void *stream)
{
    kv_status st = layer_ok(cache, layer);
    if (st != KV_OK) return st;
    if (n_new < 0) return KV_E_BAD_CONFIG;
    if (n_new == 0) return KV_OK;
    if (!k_new || !x || !w_v) return KV_E_NULL;
    const kv_config &c = cache->cfg;
    if (((uintptr_t)k_new % 16) || ((uintptr_t)x % 16) || ((uintptr_t)w_v % 16) || ((uintptr_t)v_proj % 16)) return KV_E_ALIGN;
    if (k_stride_b % 8 || k_stride_t % 8 || k_stride_h % 8 || x_stride_b % 8 || x_stride_t % 8) return KV_E_ALIGN;
    if (k_stride_h < c.head_dim || k_stride_t < 0 || k_stride_b < 0) return KV_E_BAD_CONFIG;
    if (model_dim <= 0 || model_dim % 64 || x_stride_t < model_dim || x_stride_b < 0) return KV_E_BAD_CONFIG;
    int rope = 0;
    if (rope_cos || rope_sin) {
        if (!rope_cos || !rope_sin) return KV_E_NULL;
        if (((uintptr_t)rope_cos % 16) || ((uintptr_t)rope_sin % 16)) return KV_E_ALIGN;
        if (pairing != KV_ROPE_HALF && pairing != KV_ROPE_INTERLEAVED) return KV_E_BAD_CONFIG;
        rope = pairing == KV_ROPE_HALF ? 1 : 2;
    }
    if (!compressv_supported(cache->geom[layer])) return KV_E_UNSUPPORTED;
    if (c.pool_blocks > 0 && !cache->table) return KV_E_BAD_CONFIG; // paged placement without a block table
    if ((long long)c.batch * c.n_kv_heads > 65535) return KV_E_UNSUPPORTED;
    for (int b = 0; b < c.batch; b++)
        if (cache->on(b) && (long long)cache->P(layer, b) + cache->R(layer, b) + n_new > c.max_tokens) return KV_E_CAPACITY;
    const int G = c.group_tokens, R = c.resid_cap;
    hipStream_t s = (hipStream_t)stream;
    for (int b0 = 0; b0 < c.batch;) {
        if (!cache->on(b0)) {
            b0++;
            continue;
        }
        int b1 = b0 + 1;
        while (b1 < c.batch && cache->on(b1) && cache->P(layer, b1) == cache->P(layer, b0) && cache->R(layer, b1) == cache->R(layer, b0)) b1++;
        const int r_old = cache->R(layer, b0);
        const long long total = (long long)r_old + n_new;
        const long long n_flush_tok = total / R * R;
        // ---- keys: the ordinary append, keys' side only
        AppendArgs a{};
        a.geom = cache->geom[layer];
        a.geom.table = cache->table;
        a.geom.table_stride = cache->table_stride;
        a.layer = cache->layers[layer];
        a.k_new = (const uint16_t *)k_new + (long long)b0 * k_stride_b;
        a.v_new = nullptr;
        a.stride_b = k_stride_b;
        a.stride_t = k_stride_t;
        a.stride_h = k_stride_h;
        a.n_kv_heads = c.n_kv_heads;
        a.batch = b1 - b0;
        a.b0 = b0;
        a.r_old = r_old;
        a.first_block = cache->P(layer, b0) / G;
        a.rope = rope;
        a.rope_cos = rope_cos;
        a.rope_sin = rope_sin;
        a.sides = 1;
        a.n_flush_blocks = (int)(n_flush_tok / G);
        if (n_flush_tok > 0) {
            a.copy_src = (int)(n_flush_tok - r_old);
            a.copy_dst = 0;
            a.copy_n = (int)(total - n_flush_tok);
        } else {
            a.copy_src = 0;
            a.copy_dst = r_old;
            a.copy_n = n_new;
        }
        if (a.n_flush_blocks > 0 && launch_flush(a, s) != hipSuccess) return KV_E_HIP;
        if (a.copy_n > 0 && launch_resid_copy(a, s) != hipSuccess) return KV_E_HIP;
        // ---- values: projected by the kernels that also compress them (whole blocks of this call's
        // tokens) or store them as raw rows (tokens that complete a block begun earlier, and the tail)
        ProjectArgs p{};
        p.geom = a.geom;
        p.layer = a.layer;
        p.x = (const uint16_t *)x + (long long)b0 * x_stride_b;
        p.x_stride_b = x_stride_b;
        p.x_stride_t = x_stride_t;
        p.w = (const uint16_t *)w_v;
        p.model_dim = model_dim;
        p.n_kv_heads = c.n_kv_heads;
        p.batch = b1 - b0;
        p.b0 = b0;
        p.vo_stride_h = c.head_dim;
        p.vo_stride_t = (long long)c.n_kv_heads * c.head_dim;
        p.vo_stride_b = (long long)n_new * p.vo_stride_t;
        p.v_out = v_proj ? (uint16_t *)v_proj + (long long)b0 * p.vo_stride_b : nullptr;
        auto raw_rows = [&](int t0, int n, int dst) {
            ProjectArgs q = p;
            q.mode = 1;
            q.t0 = t0;
            q.n_tok = n;
            q.n_groups = (n + 31) / 32;
            q.dst_row = dst;
            return launch_compressv(q, s) == hipSuccess;
        };
        if (n_flush_tok == 0) {
            if (!raw_rows(0, n_new, r_old)) return KV_E_HIP;
        } else {
            const int n_pre = (G - r_old % G) % G; // tokens that complete the block begun by earlier calls
            if (n_pre > 0 && !raw_rows(0, n_pre, r_old)) return KV_E_HIP;
            const int n_old_blocks = (r_old + n_pre) / G; // blocks whose rows all wait in the residual buffer now
            if (n_old_blocks > 0) {
                AppendArgs av = a;
                av.sides = 2;
                av.rope = 0;
                av.r_old = r_old + n_pre;
                av.n_flush_blocks = n_old_blocks;
                if (launch_flush(av, s) != hipSuccess) return KV_E_HIP;
            }
            const int n_new_blocks = (int)(n_flush_tok / G) - n_old_blocks;
            if (n_new_blocks > 0) {
                ProjectArgs q = p;
                q.mode = 0;
                q.t0 = n_pre;
                q.n_groups = n_new_blocks;
                q.n_tok = 32 * n_new_blocks;
                q.first_block = a.first_block + n_old_blocks;
                if (launch_compressv(q, s) != hipSuccess) return KV_E_HIP;
            }
            const int tail = (int)(total - n_flush_tok);
            if (tail > 0 && !raw_rows((int)(n_flush_tok - r_old), tail, 0)) return KV_E_HIP;
        }
        for (int b = b0; b < b1; b++) {
            cache->P(layer, b) += (int)n_flush_tok;
            cache->R(layer, b) = (int)(total - n_flush_tok);
        }
        b0 = b1;
    }
    return KV_OK;
}

kv_status kv_decode_splits(const kv_cache *cache, int32_t layer, int32_t *n_splits)
{
    kv_status st = layer_ok(cache, layer);
    if (st != KV_OK) return st;
    if (!n_splits) return KV_E_NULL;
    DecodeArgs a{};
    st = fill_decode(cache, layer, &a);
    if (st != KV_OK) return st;
    *n_splits = a.n_splits;
    return KV_OK;
}

kv_status kv_decode_bytes(const kv_cache *cache, int32_t layer, size_t *bytes)
{
    kv_status st = layer_ok(cache, layer);
    if (st != KV_OK) return st;
    if (!bytes) return KV_E_NULL;
    const kv_config &c = cache->cfg;
    const LayerGeom &g = cache->geom[layer];
    const size_t H = c.n_kv_heads, d = c.head_dim;
    size_t nb = 0, r_sum = 0; // blocks and raw tokens summed over the sequences
    for (int b = 0; b < c.batch; b++) {
        if (!cache->on(b)) continue; // a decode launch does not read the sequences that are not active
        nb += cache->P(layer, b) / c.group_tokens;
        r_sum += cache->R(layer, b);
    }
    size_t rec = 0; // bytes of a record that carry information (no padding)
    rec += (size_t)g.G * d * g.k_bits / 8;
    if (g.k_bits != 16) rec += 2 * d * 2 + (g.k_mean >= 0 ? d * 2 : 0);
    rec += (size_t)g.G * d * g.v_bits / 8;
    if (g.v_bits != 16) rec += (size_t)g.G * (d / g.Gc) * 4 + (g.v_mean >= 0 ? d * 2 : 0);
    size_t total = H * nb * rec;
    if (c.mean_mode == KV_MEAN_CROSS_HEAD) {
        size_t sides = (g.k_bits != 16) + (g.v_bits != 16);
        total += nb * sides * g.G * d * 2;
    }
    total += H * r_sum * d * 2 * 2;
    total += (size_t)c.batch * c.n_q_heads * d * (2 + 4);
    *bytes = total;
    return KV_OK;
}

kv_status kv_set_decode_path(kv_cache *cache, int32_t path)
{
    if (!cache) return KV_E_NULL;
    if (path < 0 || path > 2) return KV_E_BAD_CONFIG;
    cache->decode_path = path;
    return KV_OK;
}

kv_status kv_decode_path_used(const kv_cache *cache, int32_t layer, int32_t *path)
{
    kv_status st = layer_ok(cache, layer);
    if (st != KV_OK) return st;
    if (!path) return KV_E_NULL;
    DecodeArgs a{};
    st = fill_decode(cache, layer, &a);
    if (st != KV_OK) return st;
    if (cache->decode_path == 2 && !decode_mfma_supported(a)) return KV_E_UNSUPPORTED;
    *path = use_mfma(cache, a) ? 2 : 1;
    return KV_OK;
}

kv_status kv_set_decode_splits(kv_cache *cache, int32_t n_splits)
{
    if (!cache) return KV_E_NULL;
    if (n_splits < 0 || n_splits > kMaxSplits) return KV_E_BAD_CONFIG;
    cache->forced_splits = n_splits;
    return KV_OK;
}

kv_status kv_decode_attn_split(const kv_cache *cache, int32_t layer, const void *q,
                               void *workspace, size_t workspace_bytes, void *stream)
{
    kv_status st = layer_ok(cache, layer);
    if (st != KV_OK) return st;
    if (!q) return KV_E_NULL;
    if ((uintptr_t)q % 16) return KV_E_ALIGN;
    DecodeArgs a{};
    st = fill_decode(cache, layer, &a);
    if (st != KV_OK) return st;
    st = bind_workspace(cache, &a, workspace, workspace_bytes);
    if (st != KV_OK) return st;
    a.q = (const uint16_t *)q;
    a.out = nullptr;
    hipStream_t s = (hipStream_t)stream;
    if (cache->decode_path == 2 && !decode_mfma_supported(a)) return KV_E_UNSUPPORTED;
    hipError_t e = use_mfma(cache, a) ? launch_decode_split_mfma(a, s) : launch_decode_split_valu(a, s);
    return e == hipSuccess ? KV_OK : KV_E_HIP;
}

static kv_status merge_impl(const kv_cache *cache, int32_t layer, float *out, uint16_t *out16,
                            const void *workspace, size_t workspace_bytes, void *stream)
{
    kv_status st = layer_ok(cache, layer);
    if (st != KV_OK) return st;
    if (!out && !out16) return KV_E_NULL;
    if (((uintptr_t)out % 16) || ((uintptr_t)out16 % 16)) return KV_E_ALIGN;
    DecodeArgs a{};
    st = fill_decode(cache, layer, &a);
    if (st != KV_OK) return st;
    st = bind_workspace(cache, &a, const_cast<void *>(workspace), workspace_bytes);
    if (st != KV_OK) return st;
    a.q = nullptr;
    a.out = out;
    a.out16 = out16;
    // cross-head mean on the matrix-core path: the value mean plane's share joins the partials first
    if (a.xs && launch_xhead_values(a, (hipStream_t)stream) != hipSuccess) return KV_E_HIP;
    return launch_decode_merge(a, (hipStream_t)stream) == hipSuccess ? KV_OK : KV_E_HIP;
}

kv_status kv_decode_attn_merge(const kv_cache *cache, int32_t layer, float *out,
                               const void *workspace, size_t workspace_bytes, void *stream)
{
    if (!out) return KV_E_NULL;
    return merge_impl(cache, layer, out, nullptr, workspace, workspace_bytes, stream);
}

kv_status kv_decode_attn_merge16(const kv_cache *cache, int32_t layer, void *out16,
                                 const void *workspace, size_t workspace_bytes, void *stream)
{
    if (!out16) return KV_E_NULL;
    return merge_impl(cache, layer, nullptr, (uint16_t *)out16, workspace, workspace_bytes, stream);
}

kv_status kv_dequant(const kv_cache *cache, int32_t layer, float *k_out, float *v_out, int32_t t_cap, void *stream)
{
    kv_status st = layer_ok(cache, layer);
    if (st != KV_OK) return st;
    if (!k_out && !v_out) return KV_E_NULL;
    if (((uintptr_t)k_out % 16) || ((uintptr_t)v_out % 16)) return KV_E_ALIGN;
    const kv_config &c = cache->cfg;
    for (int b = 0; b < c.batch; b++)
        if (cache->on(b) && cache->P(layer, b) + cache->R(layer, b) > t_cap) return KV_E_CAPACITY;
    DequantArgs q{};
    st = fill_decode(cache, layer, &q.d);
    if (st != KV_OK) return st;
    q.k_out = k_out;
    q.v_out = v_out;
    q.t_cap = t_cap;
    return launch_dequant(q, (hipStream_t)stream) == hipSuccess ? KV_OK : KV_E_HIP;
}

kv_status kv_append_decode_attn_split(kv_cache *cache, int32_t layer, const void *k_new, const void *v_new,
                                      int64_t stride_b, int64_t stride_h, const void *q,
                                      void *workspace, size_t workspace_bytes, void *stream)
{
    kv_status st = layer_ok(cache, layer);
    if (st != KV_OK) return st;
    if (!k_new || !v_new || !q) return KV_E_NULL;
    const kv_config &c = cache->cfg;
    if (((uintptr_t)k_new % 16) || ((uintptr_t)v_new % 16) || ((uintptr_t)q % 16)) return KV_E_ALIGN;
    if (stride_b % 8 || stride_h % 8) return KV_E_ALIGN;
    if (stride_h < c.head_dim || stride_b < 0) return KV_E_BAD_CONFIG;
    bool flush = false; // does the token complete a block of some sequence
    for (int b = 0; b < c.batch; b++) {
        if (!cache->on(b)) continue;
        if ((long long)cache->P(layer, b) + cache->R(layer, b) + 1 > c.max_tokens) return KV_E_CAPACITY;
        if (cache->R(layer, b) + 1 == c.resid_cap) flush = true;
    }

    // the decode launch as it will look once the token is in, checked before anything is enqueued
    const std::vector<int> p_old(cache->packed.begin() + (size_t)layer * c.batch, cache->packed.begin() + (size_t)(layer + 1) * c.batch);
    const std::vector<int> r_old(cache->resid.begin() + (size_t)layer * c.batch, cache->resid.begin() + (size_t)(layer + 1) * c.batch);
    auto restore = [&] {
        for (int b = 0; b < c.batch; b++) {
            cache->P(layer, b) = p_old[b];
            cache->R(layer, b) = r_old[b];
        }
    };
    for (int b = 0; b < c.batch; b++) {
        if (!cache->on(b)) continue;
        const bool fl = r_old[b] + 1 == c.resid_cap;
        cache->P(layer, b) = fl ? p_old[b] + c.resid_cap : p_old[b];
        cache->R(layer, b) = fl ? 0 : r_old[b] + 1;
    }
    DecodeArgs a{};
    st = fill_decode(cache, layer, &a);
    const bool mfma = st == KV_OK && use_mfma(cache, a);
    if (st == KV_OK) st = bind_workspace(cache, &a, workspace, workspace_bytes);
    if (st == KV_OK && cache->decode_path == 2 && !mfma) st = KV_E_UNSUPPORTED;
    if (st != KV_OK || flush || !mfma) {
        restore();
        if (st != KV_OK) return st;
        // a block is due for compression, or the layer is served by the vector-ALU kernels:
        // the two steps run as launches of their own
        st = kv_quant_append(cache, layer, k_new, v_new, 1, stride_b, 0, stride_h, stream);
        if (st != KV_OK) return st;
        return kv_decode_attn_split(cache, layer, q, workspace, workspace_bytes, stream);
    }
    a.q = (const uint16_t *)q;
    a.out = nullptr;
    a.k_fresh = (const uint16_t *)k_new;
    a.v_fresh = (const uint16_t *)v_new;
    a.fresh_stride_b = stride_b;
    a.fresh_stride_h = stride_h;
    if (launch_decode_split_mfma(a, (hipStream_t)stream) != hipSuccess) {
        restore();
        return KV_E_HIP;
    }
    return KV_OK;
}

kv_status kv_append_decode_attn(kv_cache *cache, int32_t layer, const void *k_new, const void *v_new,
                                int64_t stride_b, int64_t stride_h, const void *q, float *out,
                                void *workspace, size_t workspace_bytes, void *stream)
{
    if (!out) return KV_E_NULL;
    if ((uintptr_t)out % 16) return KV_E_ALIGN;
    kv_status st = kv_append_decode_attn_split(cache, layer, k_new, v_new, stride_b, stride_h, q, workspace,
                                               workspace_bytes, stream);
    if (st != KV_OK) return st;
    return kv_decode_attn_merge(cache, layer, out, workspace, workspace_bytes, stream);
}

kv_status kv_decode_attn(const kv_cache *cache, int32_t layer, const void *q, float *out,
                         void *workspace, size_t workspace_bytes, void *stream)
{
    if (!out) return KV_E_NULL;
    if ((uintptr_t)out % 16) return KV_E_ALIGN;
    kv_status st = kv_decode_attn_split(cache, layer, q, workspace, workspace_bytes, stream);
    if (st != KV_OK) return st;
    return kv_decode_attn_merge(cache, layer, out, workspace, workspace_bytes, stream);
}

kv_status kv_dev_lengths_bytes(const kv_config *cfg, size_t *bytes)
{
    if (!bytes) return KV_E_NULL;
    kv_status st = check_config(cfg);
    if (st != KV_OK) return st;
    *bytes = (size_t)cfg->n_layers * dev_len_ints(cfg->batch) * sizeof(int);
    return KV_OK;
}

kv_status kv_cache_lengths_to_device(kv_cache *cache, void *dev_lengths, void *stream)
{
    if (!cache || !dev_lengths) return KV_E_NULL;
    if ((uintptr_t)dev_lengths % 16) return KV_E_ALIGN;
    const kv_config &c = cache->cfg;
    const int n = dev_len_ints(c.batch);
    cache->len_image.assign((size_t)c.n_layers * n, 0);
    for (int l = 0; l < c.n_layers; l++)
        for (int p = 0; p < 2; p++)
            for (int b = 0; b < c.batch; b++) {
                cache->len_image[(size_t)l * n + p * 2 * c.batch + 2 * b] = cache->P(l, b) / c.group_tokens;
                cache->len_image[(size_t)l * n + p * 2 * c.batch + 2 * b + 1] = cache->R(l, b);
            }
    if (note_launch(hipMemcpyAsync(dev_lengths, cache->len_image.data(), cache->len_image.size() * sizeof(int),
                                   hipMemcpyHostToDevice, (hipStream_t)stream)) != hipSuccess)
        return KV_E_HIP;
    cache->len_dev = (int *)dev_lengths;
    return KV_OK;
}

// what one decode step does to a sequence's lengths (tokens), or nothing if the sequence is full
static void step_lengths(const kv_config &c, int *packed, int *resid)
{
    const int cap = c.max_tokens / c.group_tokens * c.group_tokens;
    if (*resid >= c.resid_cap || *packed + *resid + 1 > cap) return;
    if (*resid + 1 == c.resid_cap) {
        *packed += c.resid_cap;
        *resid = 0;
    } else {
        *resid += 1;
    }
}

kv_status kv_cache_advance(kv_cache *cache, int32_t layer, int32_t n_steps)
{
    if (!cache) return KV_E_NULL;
    if (n_steps < 0) return KV_E_BAD_CONFIG;
    const kv_config &c = cache->cfg;
    if (layer < -1 || layer >= c.n_layers) return KV_E_BAD_LAYER;
    for (int l = layer < 0 ? 0 : layer; l < (layer < 0 ? c.n_layers : layer + 1); l++)
        for (int b = 0; b < c.batch; b++)
            for (int i = 0; i < n_steps; i++) step_lengths(c, &cache->P(l, b), &cache->R(l, b));
    return KV_OK;
}

kv_status kv_decode_step_dev(const kv_cache *cache, int32_t layer, const void *k_new, const void *v_new,
                             int64_t stride_b, int64_t stride_h, const void *q, float *out,
                             void *workspace, size_t workspace_bytes, void *stream)
{
    kv_status st = layer_ok(cache, layer);
    if (st != KV_OK) return st;
    if (!k_new || !v_new || !q || !out) return KV_E_NULL;
    if (!cache->len_dev) return KV_E_BAD_CONFIG; // kv_cache_lengths_to_device has not been called
    const kv_config &c = cache->cfg;
    if (((uintptr_t)k_new % 16) || ((uintptr_t)v_new % 16) || ((uintptr_t)q % 16) || ((uintptr_t)out % 16)) return KV_E_ALIGN;
    if (stride_b % 8 || stride_h % 8) return KV_E_ALIGN;
    if (stride_h < c.head_dim || stride_b < 0) return KV_E_BAD_CONFIG;
    if (!cache->active.empty()) return KV_E_UNSUPPORTED;
    if (c.pool_blocks > 0 && !cache->table) return KV_E_BAD_CONFIG; // paged placement without a block table
    if (!step_store_supported(cache->geom[layer]) || cache->decode_path == 1) return KV_E_UNSUPPORTED;

    // the launches are sized for the lengths the host knows, one step on (a recorded call is replayed
    // while the cache grows: the kernels take the true lengths from the device)
    DecodeArgs a{};
    {
        kv_cache planned = *cache; // (host state only: vectors of lengths)
        for (int b = 0; b < c.batch; b++) step_lengths(c, &planned.P(layer, b), &planned.R(layer, b));
        st = fill_decode(&planned, layer, &a);
        if (st != KV_OK) return st;
    }
    if (!use_mfma(cache, a)) return KV_E_UNSUPPORTED;
    // (mean over the heads: the form with both mean terms inside the split kernel; the kernels of the
    // other form take their lengths from the host)
    if (c.mean_mode == KV_MEAN_CROSS_HEAD && !xhead_fused(a)) return KV_E_UNSUPPORTED;
    st = bind_workspace(cache, &a, workspace, workspace_bytes);
    if (st != KV_OK) return st;
    a.ragged = 0;
    a.len_dev = cache->len_dev + (size_t)layer * dev_len_ints(c.batch);
    a.q = (const uint16_t *)q;
    a.out = out;

    AppendArgs ap{};
    ap.geom = cache->geom[layer];
    ap.geom.table = cache->table; // (paged placement: the blocks that replayed steps fill need their slots beforehand)
    ap.geom.table_stride = cache->table_stride;
    ap.layer = cache->layers[layer];
    ap.k_new = (const uint16_t *)k_new;
    ap.v_new = (const uint16_t *)v_new;
    ap.stride_b = stride_b;
    ap.stride_t = 0;
    ap.stride_h = stride_h;
    ap.n_kv_heads = c.n_kv_heads;
    ap.batch = c.batch;
    ap.b0 = 0;
    ap.r_old = c.resid_cap - 1; // a buffer that the token fills: its rows, then the caller's row
    ap.first_block = 0;
    ap.n_flush_blocks = c.resid_cap / c.group_tokens;
    ap.len_dev = a.len_dev;
    hipStream_t s = (hipStream_t)stream;
    if (launch_flush(ap, s) != hipSuccess) return KV_E_HIP; // (stores the token, too)
    if (launch_decode_split_mfma(a, s) != hipSuccess) return KV_E_HIP;
    return launch_decode_merge(a, s) == hipSuccess ? KV_OK : KV_E_HIP;
}

kv_status kv_time_next_split(void *begin_event, void *end_event)
{
    if ((begin_event == nullptr) != (end_event == nullptr)) return KV_E_NULL;
    set_split_timing_events((hipEvent_t)begin_event, (hipEvent_t)end_event);
    return KV_OK;
}

kv_status kv_stream_read_probe(const void *buf, size_t bytes, void *sink8, void *stream)
{
    if (!buf) return KV_E_NULL;
    if (((uintptr_t)buf % 16) || ((uintptr_t)sink8 % 8)) return KV_E_ALIGN;
    if (bytes < 16) return KV_E_BAD_CONFIG;
    return launch_stream_read(buf, bytes, (unsigned long long *)sink8, (hipStream_t)stream) == hipSuccess ? KV_OK : KV_E_HIP;
}

kv_status kv_decode_workspace_need(const kv_cache *cache, int32_t layer, size_t *bytes)
{
    kv_status st = layer_ok(cache, layer);
    if (st != KV_OK) return st;
    if (!bytes) return KV_E_NULL;
    DecodeArgs a{};
    st = fill_decode(cache, layer, &a);
    if (st != KV_OK) return st;
    *bytes = launch_workspace_need(cache, a);
    return KV_OK;
}

} // extern "C"

// ---- decode attention without a caller workspace: the partial results live in the device image

// Scratch for the per-split partial results of kv_decode_attn_static.  In host code this name is a
// stand-in, not a device address: the address comes from hipGetSymbolAddress, once per device.
static __device__ __align__(256) unsigned char scratch[KV_STATIC_WORKSPACE_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_lock;
void *g_scratch_ptr[kMaxDevices]; // device address of `scratch` on each device, null until first use

// Address of the current device's copy of `scratch` (null on failure; the HIP error is noted).
void *static_scratch()
{
    int dev = -1;
    if (note_launch(hipGetDevice(&dev)) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> hold(g_scratch_lock);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (note_launch(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch))) != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = p;
    }
    return g_scratch_ptr[dev];
}
} // namespace

extern "C" kv_status kv_decode_attn_static(const kv_cache *cache, int32_t layer, const void *q, float *out, void *stream)
{
    size_t need = 0;
    kv_status st = kv_decode_workspace_need(cache, layer, &need);
    if (st != KV_OK) return st;
    if (need > (size_t)KV_STATIC_WORKSPACE_BYTES) return KV_E_WORKSPACE;
    void *ws = static_scratch();
    if (!ws) return KV_E_HIP;
    return kv_decode_attn(cache, layer, q, out, ws, (size_t)KV_STATIC_WORKSPACE_BYTES, stream);
}
