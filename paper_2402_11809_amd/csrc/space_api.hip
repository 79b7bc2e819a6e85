// C ABI of the SPACE auto-correct decoding step (see include/space.h for the contract).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdlib>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <map>
#include <string>
#include <vector>

#include "../../include/space.h"
#include "space_kernels.h"

using namespace space;

struct space_layout {
    int L = 0, G = 0;
    int max_masks = 0;
    int32_t* dev = nullptr;  // [info L | rel_pos L | real_row G | n_mask G]
    LayoutDev view() const {
        LayoutDev v;
        v.info = dev;
        v.rel_pos = dev + L;
        v.real_row = dev + 2 * L;
        v.n_mask = dev + 2 * L + G;
        v.L = L;
        v.G = G;
        return v;
    }
};

namespace {

struct LayerPacked {
    PackedW qkv, o, gate_up, down;
    const uint16_t* attn_norm = nullptr;
    const uint16_t* ffn_norm = nullptr;
    bool loaded = false;
};

thread_local std::string g_init_error;

}  // namespace

// Scratch of space_sample_verify_static: the per-row lists of the two sampling-verification kernels
// (kept token ids, their probabilities, their count) and the internal copy of the accepted counts, for
// up to SPACE_STATIC_MAX_ROWS block rows.  Every GPU the library runs on holds its own copy of this
// array for the life of the process; the name below is only a host-side handle, the device address
// comes from hipGetSymbolAddress (static_scratch_address) and is what the kernels are given.
struct StaticSampleScratch {
    int32_t row_ids[SPACE_STATIC_MAX_ROWS * kMaxTopK];
    float row_probs[SPACE_STATIC_MAX_ROWS * kMaxTopK];
    int32_t row_n[SPACE_STATIC_MAX_ROWS];
    int32_t accepted_ws[SPACE_STATIC_MAX_ROWS];
};
static __device__ __align__(256) unsigned char scratch[sizeof(StaticSampleScratch)];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_dev[kMaxDevices];  // device address of `scratch` on each GPU, looked up once per GPU

// Device address of `scratch` on the current GPU; no allocation.  hipErrorInvalidDevice beyond kMaxDevices.
hipError_t static_scratch_address(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_dev[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_dev[dev] = p;
    }
    *out = g_scratch_dev[dev];
    return hipSuccess;
}

}  // namespace

struct space_ctx {
    space_config cfg{};
    std::string err;
    std::vector<void*> allocs;
    std::vector<LayerPacked> layers;
    PackedW lm;
    const uint16_t* embed = nullptr;
    const uint16_t* final_norm = nullptr;
    // scratch sized for m_max = max_batch * max_rows rows
    int m_max = 0, hd = 0, hd_kv = 0, kv_heads = 0, kt_d = 0, kt_hd = 0, kt_ffn = 0, lp_max = 0, row_tiles_max = 0;
    size_t q_plane = 0;
    int part_splits_max = 8;
    // Projections over at least wide_min_rows rows use the many-row kernel where wide_mask allows it
    // (bit 0 QKV, 1 O, 2 gate/up, 3 down, 4 LM head).  Measured at 7B shapes (all projections of a
    // layer, skinny passes -> many-row kernel, in us): 128 rows 193 -> 210 (but QKV alone 47 -> 33), 192
    // rows 205 -> 224 (QKV level), 208 rows 286 -> 238, 288 rows 296 -> 260, 384 rows 381 -> 340, 512 rows
    // 521 -> 370, 1024 rows 1015 -> 640: from the third 96-row pass on, and for QKV from the second.
    int wide_min_rows = 193, wide_min_rows_qkv = 97, wide_mask = 31;
    // How the many-row kernel cuts the rows of (projection class, row count), where space_tune_rows has
    // measured it; key = class << 32 | rows.  Without an entry: pieces of 128 rows and one for the rest.
    struct WideTuned { WideParts parts; int ksplit; };  // ksplit 0: the plan's own
    std::map<uint64_t, WideTuned> wide_parts;
    // SPACE_TUNE widecut=: a cut forced on every launch of the many-row kernel whose rows make up exactly
    // wide_cut_groups groups of two row tiles (0: none)
    WideParts wide_cut{};
    int wide_cut_groups = 0;
    // Longest context, in 32-key chunks, that a lone sequence handles with one workgroup per (head, query
    // tile); measured cross-over with the split over the key axis on a 7B-shaped model: between 1536
    // (4.09 against 4.14 ms per step) and 2048 tokens (4.26 against 4.25).
    // SPACE_TUNE="attn=N" overrides (0: always split over the key axis).
    int head_attn_max_chunks = 36;
    int wide_ks = 0;      // SPACE_TUNE wideks=N: partial sums over the contraction in the many-row kernel (0: cost model / measurement)
    size_t part_stride = 0;
    int part_ld = 0;
    float* x = nullptr;
    uint16_t* xn = nullptr;
    float* part = nullptr;
    uint16_t *q = nullptr, *kblk = nullptr, *vblk = nullptr, *attn_out = nullptr, *h = nullptr;
    float *o_part = nullptr, *ml_part = nullptr;
    int attn_wg_max = 1;
    float* arg_val = nullptr;
    int32_t* arg_idx = nullptr;
    int arg_groups = 0;
    float *cos_t = nullptr, *sin_t = nullptr;      // rotary factors of the rows of the current block
    float *cos_tab = nullptr, *sin_tab = nullptr;  // ... of every position 0 .. n_pos-1 (filled once)
    int n_pos = 0;
    int32_t *pos = nullptr, *argmax_ws = nullptr, *accepted_ws = nullptr, *faults = nullptr;
    int32_t *row_ids = nullptr, *row_n = nullptr;  // sampling verification: kept ids / count of every row
    float* row_probs = nullptr;
    float* loss_ws = nullptr;  // per-row loss terms when the caller does not ask for them
    std::vector<space_layout*> layouts;
    const void* staged_kv = nullptr;  // kv->len of the cache (view) the last step staged a block on
    int staged_groups = 0;
    // per-class launch timing (measurement hook)
    uint32_t timing_mask = 0;
    std::vector<hipEvent_t> ev_start, ev_stop;
    std::vector<int> ev_class;
    size_t ev_used = 0;
    double ev_overhead_ms = 0.0;  // what an empty start/stop bracket measures
};

namespace {

int fail(space_ctx* ctx, int code, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    if (ctx) ctx->err = buf; else g_init_error = buf;
    return code;
}

#define HIP_TRY(ctx, expr)                                                                        \
    do {                                                                                          \
        hipError_t e_ = (expr);                                                                   \
        if (e_ != hipSuccess) return fail(ctx, SPACE_EHIP, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

template <typename T>
int dev_alloc(space_ctx* ctx, T** p, size_t count, bool zero) {
    void* raw = nullptr;
    const size_t bytes = count * sizeof(T);
    if (hipMalloc(&raw, bytes ? bytes : 16) != hipSuccess) {
        (void)hipGetLastError();
        return fail(ctx, SPACE_ENOMEM, "device allocation of %zu bytes failed", bytes);
    }
    ctx->allocs.push_back(raw);
    if (zero && bytes) HIP_TRY(ctx, hipMemset(raw, 0, bytes));
    *p = (T*)raw;
    return SPACE_OK;
}

// Tiling of one projection: tiles per wave and splits of the contraction.  Few wide waves keep the
// activation re-reads low (each wave reads every activation tile of its contraction range once per
// r_pack weight tiles); the splits keep enough waves streaming when W has few rows.
// SPACE_TUNE="qkv=8:2,o=4:4,gu=8:1,dn=4:4,lm=8:1" overrides (developer knob).
void plan_matrix(PackedW* w, const char* name, int n, int k, bool may_split) {
    const int n_tiles = ceil_div(n, kTileN), k_tiles = ceil_div(k, kTileK);
    // Cost model fitted on MI355X: a workgroup streams r * lq weight tiles per wave plus the 6
    // activation planes of each contraction tile through one CU, whose fill rate is the limit;
    // workgroups beyond one per CU (256) run in a second round; every doubling of the split adds
    // partial sums to write and re-read.
    int r = 4, s = 1;
    double best = 1e30;
    for (int rc : {8, 6, 4, 2}) {
        for (int sc = 1; sc <= (may_split ? 8 : 1); sc *= 2) {
            const int lq = ceil_div(k_tiles, 4 * sc);
            if (sc > 1 && lq < 6) continue;
            const int wgs = ceil_div(n_tiles, rc) * sc;
            double cost = (double)ceil_div(wgs, 256) * lq * (rc + 6.0);
            for (int t = sc; t > 1; t /= 2) cost *= 1.08;
            if (cost < best) { best = cost; r = rc; s = sc; }
        }
    }
    if (const char* e = getenv("SPACE_TUNE")) {
        std::string key = std::string(name) + "=";
        if (const char* p = strstr(e, key.c_str())) {
            int rr = 0, ss = 0;
            if (sscanf(p + key.size(), "%d:%d", &rr, &ss) == 2 && (rr == 2 || rr == 4 || rr == 6 || rr == 8) && ss >= 1 && ss <= 8) {
                r = rr;
                if (may_split) s = ss;
            }
        }
    }
    plan_packed(w, n, k, r, s);
}

int pack_into(space_ctx* ctx, PackedW* w, const void* s0, int n0, const void* s1, int n1, const void* s2, int n2,
              int interleave) {
    uint8_t* buf = nullptr;
    int rc = dev_alloc(ctx, &buf, w->bytes(), false);
    if (rc) return rc;
    HIP_TRY(ctx, launch_pack(s0, n0, s1, n1, s2, n2, interleave, *w, buf, nullptr));
    w->data = buf;
    return SPACE_OK;
}

int copy_dev(space_ctx* ctx, const uint16_t** dst, const void* src, size_t count) {
    uint16_t* p = nullptr;
    int rc = dev_alloc(ctx, &p, count, false);
    if (rc) return rc;
    HIP_TRY(ctx, hipMemcpy(p, src, count * sizeof(uint16_t), hipMemcpyDeviceToDevice));
    *dst = p;
    return SPACE_OK;
}

// Packs the canonical tensors of layer l into library-owned memory (the plan of every matrix exists).
int load_layer(space_ctx* ctx, int l, const space_layer_weights& lw) {
    const space_config& c = ctx->cfg;
    const int d = c.d_model, hd = ctx->hd, hd_kv = ctx->hd_kv, f = c.ffn;
    if (!lw.attn_norm || !lw.wq || !lw.wk || !lw.wv || !lw.wo || !lw.ffn_norm || !lw.w_gate || !lw.w_up || !lw.w_down)
        return fail(ctx, SPACE_EINVAL, "layer %d: null weight pointer", l);
    LayerPacked& lp = ctx->layers[l];
    if (lp.loaded) return fail(ctx, SPACE_EINVAL, "layer %d was loaded before", l);
    int rc;
    if ((rc = pack_into(ctx, &lp.qkv, lw.wq, hd, lw.wk, hd_kv, lw.wv, hd_kv, 0))) return rc;
    if ((rc = pack_into(ctx, &lp.o, lw.wo, d, nullptr, 0, nullptr, 0, 0))) return rc;
    if ((rc = pack_into(ctx, &lp.gate_up, lw.w_gate, f, lw.w_up, f, nullptr, 0, 1))) return rc;
    if ((rc = pack_into(ctx, &lp.down, lw.w_down, d, nullptr, 0, nullptr, 0, 0))) return rc;
    if ((rc = copy_dev(ctx, &lp.attn_norm, lw.attn_norm, d))) return rc;
    if ((rc = copy_dev(ctx, &lp.ffn_norm, lw.ffn_norm, d))) return rc;
    lp.loaded = true;
    return SPACE_OK;
}

int check_config(const space_config* c) {
    if (c->n_layers < 1 || c->d_model < 32 || c->n_heads < 1 || c->ffn < 1 || c->vocab < 1 || c->max_batch < 1 ||
        c->max_rows < 1)
        return fail(nullptr, SPACE_EINVAL, "space_config: sizes must be positive");
    if (c->head_dim != 64 && c->head_dim != 128)
        return fail(nullptr, SPACE_ESHAPE, "head_dim %d unsupported (64 or 128)", c->head_dim);
    if (c->d_model % 32 || (c->n_heads * c->head_dim) % 32)
        return fail(nullptr, SPACE_ESHAPE, "d_model and n_heads*head_dim must be multiples of 32");
    if (c->n_kv_heads < 0 || (c->n_kv_heads > 0 && c->n_heads % c->n_kv_heads))
        return fail(nullptr, SPACE_ESHAPE, "n_kv_heads %d must be 0 or divide n_heads %d", c->n_kv_heads, c->n_heads);
    if (c->d_model > 8192) return fail(nullptr, SPACE_ESHAPE, "d_model %d > 8192 unsupported", c->d_model);
    if (c->max_ctx < kAttnKeys) return fail(nullptr, SPACE_EINVAL, "max_ctx %d < %d", c->max_ctx, kAttnKeys);
    if (c->max_rows > kMaxBlockRows)
        return fail(nullptr, SPACE_ESHAPE, "max_rows %d > %d unsupported", c->max_rows, kMaxBlockRows);
    if (!(c->rms_eps > 0.f) || !(c->rope_base > 1.f)) return fail(nullptr, SPACE_EINVAL, "bad rms_eps / rope_base");
    return SPACE_OK;
}

int init_impl(space_ctx* ctx, const space_weights* w) {
    const space_config& c = ctx->cfg;
    const int d = c.d_model, hd = c.n_heads * c.head_dim, f = c.ffn;
    ctx->hd = hd;
    ctx->kv_heads = c.n_kv_heads > 0 ? c.n_kv_heads : c.n_heads;
    ctx->hd_kv = ctx->kv_heads * c.head_dim;
    const int hd_kv = ctx->hd_kv;
    ctx->m_max = c.max_batch * c.max_rows;
    ctx->row_tiles_max = ceil_div(ctx->m_max, 16);
    ctx->q_plane = (size_t)c.max_batch * c.n_heads * c.max_rows * c.head_dim;
    ctx->lp_max = round_up(c.max_rows, kAttnKeys);
    int rc;
    ctx->layers.resize(c.n_layers);
    for (int l = 0; l < c.n_layers; ++l) {
        const space_layer_weights& lw = w->layers[l];
        LayerPacked& lp = ctx->layers[l];
        plan_matrix(&lp.qkv, "qkv", hd + 2 * hd_kv, d, true);
        plan_matrix(&lp.o, "o", d, hd, true);
        plan_matrix(&lp.gate_up, "gu", 2 * round_up(f, kTileN), d, false);
        plan_matrix(&lp.down, "dn", d, f, true);
        const bool none = !lw.attn_norm && !lw.wq && !lw.wk && !lw.wv && !lw.wo && !lw.ffn_norm && !lw.w_gate &&
                          !lw.w_up && !lw.w_down;
        if (none) continue;  // handed over later with space_load_layer
        if ((rc = load_layer(ctx, l, lw))) return rc;
    }
    plan_matrix(&ctx->lm, "lm", c.vocab, d, false);
    if ((rc = pack_into(ctx, &ctx->lm, w->lm_head, c.vocab, nullptr, 0, nullptr, 0, 0))) return rc;
    // contraction tiles the activation buffers must cover (the packed matrices pad their ranges)
    const LayerPacked& l0 = ctx->layers[0];
    ctx->kt_d = std::max(std::max(l0.qkv.k_tiles_pad(), l0.gate_up.k_tiles_pad()), ctx->lm.k_tiles_pad());
    ctx->kt_hd = l0.o.k_tiles_pad();
    ctx->kt_ffn = l0.down.k_tiles_pad();
    if ((rc = copy_dev(ctx, &ctx->embed, w->embed, (size_t)(c.vocab + 1) * d))) return rc;
    if ((rc = copy_dev(ctx, &ctx->final_norm, w->final_norm, d))) return rc;

    const size_t M = ctx->m_max;
    const int nmax = hd + 2 * hd_kv > d ? hd + 2 * hd_kv : d;
    ctx->part_ld = nmax;
    ctx->part_stride = M * nmax;
    ctx->arg_groups = gemm_groups(ctx->lm, 2);
    int max_splits = 1;
    for (const PackedW* pw : {&l0.qkv, &l0.o, &l0.down}) max_splits = std::max(max_splits, pw->splits);
    if (const char* e = getenv("SPACE_TUNE")) {
        int n = 0;
        if (const char* p = strstr(e, "attn=")) {
            if (sscanf(p + 5, "%d", &n) == 1 && n >= 0) ctx->head_attn_max_chunks = n;
        }
        if (const char* p = strstr(e, "wideks=")) {
            if (sscanf(p + 7, "%d", &n) == 1 && n >= 0 && n <= 4) ctx->wide_ks = n;
        }
        if (const char* p = strstr(e, "wide=")) {
            if (sscanf(p + 5, "%d", &n) == 1 && n >= 0) ctx->wide_min_rows = ctx->wide_min_rows_qkv = n;
        }
        if (const char* p = strstr(e, "widemask=")) {
            if (sscanf(p + 9, "%d", &n) == 1 && n >= 0) ctx->wide_mask = n;
        }
        if (const char* p = strstr(e, "widecut=")) {
            WideParts w{};
            if (sscanf(p + 8, "%d:%d:%d:%d:%d", &w.count[0], &w.count[1], &w.count[2], &w.count[3], &w.by_size) == 5 &&
                w.count[0] >= 0 && w.count[1] >= 0 && w.count[2] >= 0 && w.count[3] >= 0 && (w.by_size == 0 || w.by_size == 1)) {
                ctx->wide_cut = w;
                ctx->wide_cut_groups = 4 * w.count[0] + 3 * w.count[1] + 2 * w.count[2] + w.count[3];
            }
        }
    }
    if ((ctx->wide_min_rows > 0 && ctx->m_max >= ctx->wide_min_rows) || (ctx->wide_min_rows_qkv > 0 && ctx->m_max >= ctx->wide_min_rows_qkv))
        max_splits = std::max(max_splits, 4);
    ctx->part_splits_max = max_splits;
    const size_t plane_tile = 2 * 64 * 8;  // hi + lo plane of one 16 x 32 activation tile, in elements
    const size_t rt = ctx->row_tiles_max;
    const size_t bh = (size_t)c.max_batch * c.n_heads;
    if ((rc = dev_alloc(ctx, &ctx->x, M * d, true))) return rc;
    if ((rc = dev_alloc(ctx, &ctx->xn, rt * ctx->kt_d * plane_tile, true))) return rc;
    if ((rc = dev_alloc(ctx, &ctx->part, ctx->part_stride * ctx->part_splits_max, true))) return rc;
    if ((rc = dev_alloc(ctx, &ctx->q, 2 * ctx->q_plane, true))) return rc;
    // block K/V staging: one slice per head, or one per (head, query tile) on the fused path
    const size_t stage_rows = std::max<size_t>(ctx->lp_max, (size_t)(kHeadAttnMaxRows / 16) * round_up(kHeadAttnMaxRows, kAttnKeys));
    if ((rc = dev_alloc(ctx, &ctx->kblk, bh * stage_rows * c.head_dim, true))) return rc;
    if ((rc = dev_alloc(ctx, &ctx->vblk, bh * stage_rows * c.head_dim, true))) return rc;
    if ((rc = dev_alloc(ctx, &ctx->attn_out, rt * ctx->kt_hd * plane_tile, true))) return rc;
    if ((rc = dev_alloc(ctx, &ctx->h, rt * ctx->kt_ffn * plane_tile, true))) return rc;
    // partial attention outputs: workgroups along the key axis x rows, at its worst over the block lengths
    // (the step launches with at least n_heads * query groups streams, more with a batch)
    size_t wg_rows = 1;
    for (int L = 1; L <= c.max_rows; ++L) {
        const int wg = attention_workgroups(c.max_ctx, L, c.n_heads * ceil_div(ceil_div(L, 16), 3));
        wg_rows = std::max(wg_rows, (size_t)wg * L);
        ctx->attn_wg_max = std::max(ctx->attn_wg_max, wg);
    }
    if ((rc = dev_alloc(ctx, &ctx->o_part, bh * wg_rows * c.head_dim, true))) return rc;
    if ((rc = dev_alloc(ctx, &ctx->ml_part, bh * wg_rows * 2, true))) return rc;
    if ((rc = dev_alloc(ctx, &ctx->arg_val, M * ctx->arg_groups, true))) return rc;
    if ((rc = dev_alloc(ctx, &ctx->arg_idx, M * ctx->arg_groups, true))) return rc;
    if ((rc = dev_alloc(ctx, &ctx->cos_t, M * (c.head_dim / 2), true))) return rc;
    if ((rc = dev_alloc(ctx, &ctx->sin_t, M * (c.head_dim / 2), true))) return rc;
    ctx->n_pos = c.max_ctx + c.max_rows + 1;
    if ((rc = dev_alloc(ctx, &ctx->cos_tab, (size_t)ctx->n_pos * (c.head_dim / 2), false))) return rc;
    if ((rc = dev_alloc(ctx, &ctx->sin_tab, (size_t)ctx->n_pos * (c.head_dim / 2), false))) return rc;
    HIP_TRY(ctx, launch_rope_table(ctx->cos_tab, ctx->sin_tab, ctx->n_pos, c.head_dim, c.rope_base, nullptr));
    if ((rc = dev_alloc(ctx, &ctx->pos, M, true))) return rc;
    if ((rc = dev_alloc(ctx, &ctx->argmax_ws, M, true))) return rc;
    if ((rc = dev_alloc(ctx, &ctx->accepted_ws, (size_t)c.max_batch, true))) return rc;
    if ((rc = dev_alloc(ctx, &ctx->row_ids, M * kMaxTopK, true))) return rc;
    if ((rc = dev_alloc(ctx, &ctx->row_probs, M * kMaxTopK, true))) return rc;
    if ((rc = dev_alloc(ctx, &ctx->row_n, M, true))) return rc;
    if ((rc = dev_alloc(ctx, &ctx->loss_ws, M, true))) return rc;
    if ((rc = dev_alloc(ctx, &ctx->faults, (size_t)4, true))) return rc;
    {
        void* p = nullptr;  // space_sample_verify_static: resolve its scratch on this GPU now, not under a capture
        HIP_TRY(ctx, static_scratch_address(&p));
    }
    HIP_TRY(ctx, hipDeviceSynchronize());
    return SPACE_OK;
}

void free_events(space_ctx* ctx) {
    for (hipEvent_t e : ctx->ev_start) (void)hipEventDestroy(e);
    for (hipEvent_t e : ctx->ev_stop) (void)hipEventDestroy(e);
    ctx->ev_start.clear();
    ctx->ev_stop.clear();
    ctx->ev_class.clear();
    ctx->ev_used = 0;
    ctx->timing_mask = 0;
}

// brackets the launches of one kernel class with events when that class is being timed
struct TimedScope {
    space_ctx* ctx;
    hipStream_t s;
    long slot = -1;
    TimedScope(space_ctx* c, int cls, hipStream_t st) : ctx(c), s(st) {
        if ((c->timing_mask >> cls) & 1u) {
            if (c->ev_used < c->ev_start.size()) {
                slot = (long)c->ev_used++;
                c->ev_class[slot] = cls;
                (void)hipEventRecord(c->ev_start[slot], s);
            }
        }
    }
    ~TimedScope() {
        if (slot >= 0) (void)hipEventRecord(ctx->ev_stop[slot], s);
    }
};

void free_ctx(space_ctx* ctx) {
    free_events(ctx);
    for (space_layout* l : ctx->layouts) {
        if (l->dev) (void)hipFree(l->dev);
        delete l;
    }
    for (void* p : ctx->allocs) (void)hipFree(p);
    delete ctx;
}

// One projection over all m rows.  Few rows: the weight-streaming kernel (passes of at most 96 rows
// inside one launch); many rows: the kernel that shares the activation planes through LDS.
// *splits_used = number of partial sums written to out (EPI_F32) / of per-row argmax partials' groups
// (EPI_ARGMAX: *groups_used).
int run_gemm(space_ctx* ctx, const PackedW& w, GemmEpilogue epi, const uint16_t* x, int m, float* out, int ldo,
             size_t split_stride, uint16_t* h, int ffn, float* logits, hipStream_t s, int* splits_used = nullptr,
             int* groups_used = nullptr, int wide_from = 0, int cls = -1, const WideParts* force_parts = nullptr,
             int force_ksplit = 0) {
    const int pass_rows = 16 * kMaxRowTiles;
    GemmLaunch g{};
    g.w = w;
    g.x = x;
    g.xs = xt_shape(m);
    g.row_tile0 = 0;
    g.m = m;
    g.passes = ceil_div(m, pass_rows);
    g.tiles_per_wave = gemm_tiles_per_wave(w, m);
    g.ldo = ldo;
    g.split_stride = split_stride;
    if (epi == EPI_F32) g.out = out;
    if (epi == EPI_SWIGLU) {
        g.h = h;
        g.ffn = ffn;
    }
    if (epi == EPI_ARGMAX) {
        g.out = logits;
        g.arg_val = ctx->arg_val;
        g.arg_idx = ctx->arg_idx;
        g.arg_groups = ctx->arg_groups;
    }
    if (wide_from > 0 && m >= wide_from) {  // wide_from: fewest rows for the many-row kernel, 0 = never
        // The cut of the rows changes no result, only the time; the number of partial sums over the
        // contraction (measured too, for the plain-sum projections) changes the order of the fp32 sums.
        const space_ctx::WideTuned* tuned = nullptr;
        if (!force_parts && cls >= 0 && !(ctx->wide_cut_groups > 0 && ctx->wide_cut_groups == ceil_div(ceil_div(m, 16), 2))) {
            const auto it = ctx->wide_parts.find(((uint64_t)cls << 32) | (uint32_t)m);
            if (it != ctx->wide_parts.end()) tuned = &it->second;
        }
        WidePlan p = plan_gemm_wide(w, m, epi, ctx->part_splits_max,
                                    force_parts ? force_ksplit : ctx->wide_ks > 0 ? ctx->wide_ks : tuned ? tuned->ksplit : 0);
        if (force_parts) {
            p.parts = *force_parts;
        } else if (tuned) {
            p.parts = tuned->parts;
        } else if (ctx->wide_cut_groups > 0 && ctx->wide_cut_groups == ceil_div(ceil_div(m, 16), 2)) {
            p.parts = ctx->wide_cut;
        }
        if (splits_used) *splits_used = p.ksplit;
        if (groups_used) *groups_used = p.n_groups;
        HIP_TRY(ctx, launch_gemm_wide(g, p, epi, s));
        return SPACE_OK;
    }
    if (splits_used) *splits_used = w.splits;
    if (groups_used) *groups_used = gemm_groups(w, g.tiles_per_wave);
    HIP_TRY(ctx, launch_gemm(g, epi, s));
    return SPACE_OK;
}

}  // namespace

extern "C" {

const char* space_last_error(const space_ctx* ctx) { return ctx ? ctx->err.c_str() : g_init_error.c_str(); }

int space_init(const space_config* cfg, const space_weights* weights, space_ctx** out) {
    if (out) *out = nullptr;
    if (!cfg || !weights || !out) return fail(nullptr, SPACE_EINVAL, "space_init: null argument");
    if (!weights->embed || !weights->final_norm || !weights->lm_head || !weights->layers)
        return fail(nullptr, SPACE_EINVAL, "space_init: null weight pointer");
    int rc = check_config(cfg);
    if (rc) return rc;
    space_ctx* ctx = new (std::nothrow) space_ctx();
    if (!ctx) return fail(nullptr, SPACE_ENOMEM, "host allocation failed");
    ctx->cfg = *cfg;
    rc = init_impl(ctx, weights);
    if (rc) {
        g_init_error = ctx->err;
        free_ctx(ctx);
        return rc;
    }
    *out = ctx;
    return SPACE_OK;
}

int space_load_layer(space_ctx* ctx, int32_t layer, const space_layer_weights* weights) {
    if (!ctx) return SPACE_EINVAL;
    if (!weights) return fail(ctx, SPACE_EINVAL, "space_load_layer: null argument");
    if (layer < 0 || layer >= ctx->cfg.n_layers) return fail(ctx, SPACE_EINVAL, "space_load_layer: no layer %d", layer);
    const int rc = load_layer(ctx, layer, *weights);
    if (rc) return rc;
    HIP_TRY(ctx, hipDeviceSynchronize());  // the caller may free its tensors when this returns
    return SPACE_OK;
}

void space_destroy(space_ctx* ctx) {
    if (!ctx) return;
    (void)hipDeviceSynchronize();
    free_ctx(ctx);
}

int space_layout_create(space_ctx* ctx, int32_t n_rows, const uint8_t* is_mask, const int32_t* group,
                        space_layout** out) {
    if (out) *out = nullptr;
    if (!ctx) return SPACE_EINVAL;
    if (!is_mask || !group || !out || n_rows < 1) return fail(ctx, SPACE_EINVAL, "space_layout_create: bad argument");
    if (n_rows > ctx->cfg.max_rows)
        return fail(ctx, SPACE_ECAPACITY, "layout of %d rows exceeds max_rows %d", n_rows, ctx->cfg.max_rows);
    const int L = n_rows;
    if (is_mask[0] || group[0] != 0) return fail(ctx, SPACE_EINVAL, "layout: row 0 must be the non-mask row of group 0");
    std::vector<int32_t> info(L), rel(L), real_row, n_mask;
    for (int r = 0; r < L; ++r) {
        if (is_mask[r] > 1) return fail(ctx, SPACE_EINVAL, "layout: is_mask[%d] not 0/1", r);
        if (!is_mask[r]) {
            if (group[r] != (int)real_row.size())
                return fail(ctx, SPACE_EINVAL, "layout: row %d starts group %d, expected %d", r, group[r],
                            (int)real_row.size());
            real_row.push_back(r);
            n_mask.push_back(0);
            rel[r] = group[r];  // visible in block: the non-mask rows of groups 0..g
        } else {
            if (group[r] != (int)real_row.size() - 1)
                return fail(ctx, SPACE_EINVAL, "layout: mask row %d is in group %d, expected %d", r, group[r],
                            (int)real_row.size() - 1);
            n_mask.back() += 1;
            rel[r] = group[r] + n_mask.back();  // ... plus the masks of its own group up to itself
        }
        info[r] = (group[r] << 1) | (is_mask[r] ? 1 : 0);
    }
    space_layout* lay = new (std::nothrow) space_layout();
    if (!lay) return fail(ctx, SPACE_ENOMEM, "host allocation failed");
    lay->L = L;
    lay->G = (int)real_row.size();
    for (int m : n_mask) lay->max_masks = m > lay->max_masks ? m : lay->max_masks;
    std::vector<int32_t> all;
    all.insert(all.end(), info.begin(), info.end());
    all.insert(all.end(), rel.begin(), rel.end());
    all.insert(all.end(), real_row.begin(), real_row.end());
    all.insert(all.end(), n_mask.begin(), n_mask.end());
    if (hipMalloc((void**)&lay->dev, all.size() * sizeof(int32_t)) != hipSuccess) {
        (void)hipGetLastError();
        delete lay;
        return fail(ctx, SPACE_ENOMEM, "device allocation failed");
    }
    if (hipMemcpy(lay->dev, all.data(), all.size() * sizeof(int32_t), hipMemcpyHostToDevice) != hipSuccess) {
        (void)hipFree(lay->dev);
        delete lay;
        return fail(ctx, SPACE_EHIP, "layout upload failed");
    }
    ctx->layouts.push_back(lay);
    *out = lay;
    return SPACE_OK;
}

void space_layout_destroy(space_ctx* ctx, space_layout* layout) {
    if (!ctx || !layout) return;
    for (size_t i = 0; i < ctx->layouts.size(); ++i) {
        if (ctx->layouts[i] == layout) {
            ctx->layouts.erase(ctx->layouts.begin() + i);
            (void)hipDeviceSynchronize();
            if (layout->dev) (void)hipFree(layout->dev);
            delete layout;
            return;
        }
    }
}

size_t space_kv_bytes(const space_config* cfg, int32_t batch, int32_t capacity) {
    if (!cfg || batch < 1 || capacity < kAttnKeys || capacity % kAttnKeys) return 0;
    const int kvh = cfg->n_kv_heads > 0 ? cfg->n_kv_heads : cfg->n_heads;
    return (size_t)cfg->n_layers * batch * kvh * capacity * cfg->head_dim * sizeof(uint16_t);
}

size_t space_kv_pool_bytes(const space_config* cfg, int32_t n_pages) {
    if (!cfg || n_pages < 1) return 0;
    const int kvh = cfg->n_kv_heads > 0 ? cfg->n_kv_heads : cfg->n_heads;
    return (size_t)cfg->n_layers * n_pages * kvh * kAttnKeys * cfg->head_dim * sizeof(uint16_t);
}

static int check_kv(space_ctx* ctx, const space_kv* kv) {
    if (!kv || !kv->k || !kv->v || !kv->len) return fail(ctx, SPACE_EINVAL, "space_kv: null pointer");
    if (kv->block_table && (kv->table_stride < 1 || kv->n_pages < 1 || kv->capacity != kv->table_stride * kAttnKeys))
        return fail(ctx, SPACE_EINVAL, "paged space_kv: table_stride %d, n_pages %d, capacity %d (must be 32 * table_stride)",
                    kv->table_stride, kv->n_pages, kv->capacity);
    if (kv->batch < 1 || kv->batch > ctx->cfg.max_batch)
        return fail(ctx, SPACE_ECAPACITY, "kv batch %d outside 1..max_batch %d", kv->batch, ctx->cfg.max_batch);
    if (kv->capacity < kAttnKeys || kv->capacity % kAttnKeys)
        return fail(ctx, SPACE_EINVAL, "kv capacity %d must be a positive multiple of %d", kv->capacity, kAttnKeys);
    if (kv->capacity > ctx->cfg.max_ctx)
        return fail(ctx, SPACE_ECAPACITY, "kv capacity %d exceeds max_ctx %d", kv->capacity, ctx->cfg.max_ctx);
    return SPACE_OK;
}

int space_kv_reset(space_ctx* ctx, space_kv* kv, void* stream) {
    if (!ctx) return SPACE_EINVAL;
    int rc = check_kv(ctx, kv);
    if (rc) return rc;
    hipStream_t s = (hipStream_t)stream;
    const size_t bytes = kv->block_table ? space_kv_pool_bytes(&ctx->cfg, kv->n_pages)
                                         : space_kv_bytes(&ctx->cfg, kv->batch, kv->capacity);
    HIP_TRY(ctx, launch_fill_zero(kv->k, bytes, s));
    HIP_TRY(ctx, launch_fill_zero(kv->v, bytes, s));
    HIP_TRY(ctx, launch_fill_zero(kv->len, sizeof(int32_t) * kv->batch, s));
    kv->host_len_bound = 0;
    if (ctx->staged_kv == kv->len) ctx->staged_kv = nullptr;
    return SPACE_OK;
}

}  // extern "C"

namespace {

// The decoder over one block per sequence, with (out != nullptr) or without the LM head and the
// verification behind it.
int step_impl(space_ctx* ctx, const int32_t* tokens, const space_layout* layout, const space_layout* next_layout,
              space_kv* kv, const space_step_out* out, void* stream) {
    const char* who = out ? "space_step" : "space_prefill";
    int rc = check_kv(ctx, kv);
    if (rc) return rc;
    const space_config& c = ctx->cfg;
    const int B = kv->batch, L = layout->L, G = layout->G, M = B * L;
    if (M > ctx->m_max) return fail(ctx, SPACE_ECAPACITY, "%s: %d x %d rows exceed max_batch * max_rows = %d", who, B, L, ctx->m_max);
    if (out && L > 16 * kMaxRowTiles)
        return fail(ctx, SPACE_ESHAPE, "space_step: blocks of more than %d rows only through space_prefill", 16 * kMaxRowTiles);
    if (out && out->next_tokens && next_layout && next_layout->L > 16 * kMaxRowTiles)
        return fail(ctx, SPACE_ESHAPE, "space_step: next_layout has %d rows, the verification assembles blocks of at most %d",
                    next_layout->L, 16 * kMaxRowTiles);
    if (kv->host_len_bound < 0 || kv->host_len_bound + G > kv->capacity)
        return fail(ctx, SPACE_ECAPACITY, "cache bound %d + %d groups exceeds capacity %d", kv->host_len_bound, G,
                    kv->capacity);
    for (int l = 0; l < c.n_layers; ++l)
        if (!ctx->layers[l].loaded) return fail(ctx, SPACE_EINVAL, "%s: layer %d has no weights yet (space_load_layer)", who, l);
    if (out) {
        if (out->new_cands && out->max_cands < 1) return fail(ctx, SPACE_EINVAL, "space_step: max_cands < 1");
        if (out->emit && (!out->emit_len || out->emit_cap < 1)) return fail(ctx, SPACE_EINVAL, "space_step: emit without emit_len/cap");
        if (out->eos_id >= 0 && (!out->emit || !out->finished)) return fail(ctx, SPACE_EINVAL, "space_step: eos_id needs emit and finished");
    }
    hipStream_t s = (hipStream_t)stream;
    const LayoutDev lay = layout->view();
    const int d = c.d_model, hd = ctx->hd, dh = c.head_dim;
    const int Lp = round_up(L, kAttnKeys);

    const XtShape xs = xt_shape(M);
    {
        TimedScope ts(ctx, SPACE_K_EMBED, s);
        HIP_TRY(ctx, launch_embed(tokens, ctx->embed, c.vocab, d, lay, kv->len, B, ctx->cos_tab, ctx->sin_tab, ctx->n_pos, dh,
                                  ctx->x, ctx->pos, ctx->cos_t, ctx->sin_t, ctx->faults, ctx->layers[0].attn_norm, c.rms_eps,
                                  ctx->xn, xs, s));
    }
    // the real lengths live on the device; the grid covers the host-side upper bound
    const int attn_chunks = ceil_div(kv->host_len_bound, kAttnKeys) + ceil_div(L, kAttnKeys);
    const int attn_streams = B * c.n_heads * ceil_div(ceil_div(L, 16), 3);
    const int attn_wg = attention_workgroups(kv->host_len_bound, L, attn_streams);
    const size_t kv_layer = kv->block_table ? (size_t)kv->n_pages * ctx->kv_heads * kAttnKeys * dh
                                            : (size_t)B * ctx->kv_heads * kv->capacity * dh;
    KvPaging paging;
    paging.table = kv->block_table;
    paging.table_stride = kv->table_stride;
    paging.n_pages = kv->n_pages;
    // One workgroup per head (rotary, store and attention fused) while the context is short enough
    // for a single CU to get through a head's keys; the split over the key axis beyond.
    // (with one query tile and at least a workgroup per CU it also wins at any length; with several query
    // tiles every tile's workgroup would read the head's K/V again, which long contexts do not forgive)
    // In a batch the kernel with one workgroup per (sequence, head, query tile) puts several workgroups on
    // a CU, each of which stages and reads the head's keys again, and beyond 256 workgroups it runs in two
    // rounds.  Measured against the split (7B, k = 5, us per layer at 256 / 512 / 1024 cached positions):
    // 2 sequences 9.0 / 13.3 / 22.7 against 15.4 / 19.2 / 25.3; 3 sequences (288 workgroups) 22.4 / 30.7 /
    // 44.0 against 20.1 / 24.2 / 31.5; 4 sequences 17.2 / 27.8 / 41.6 against 20.9 / 26.2 / 32.9; 6 sequences
    // lose at any length.  So: beyond one workgroup per CU only up to 12 chunks (the block's own two and
    // about 320 cached positions), beyond two per CU never.
    const long long head_wgs = (long long)B * c.n_heads * ceil_div(L, 16);
    long long head_chunks = ctx->head_attn_max_chunks;
    if (head_chunks < 1000000) {  // (1000000 and more: the developer knob that forces this kernel)
        if (head_wgs > 512) head_chunks = 0;
        else if (head_wgs > 256) head_chunks = std::min<long long>(head_chunks, 12);
    }
    const bool head_attn = L <= kHeadAttnMaxRows && ctx->head_attn_max_chunks > 0 &&
                           (attn_chunks <= head_chunks || (L <= 16 && B * c.n_heads >= 256));

    for (int l = 0; l < c.n_layers; ++l) {
        const LayerPacked& lp = ctx->layers[l];
        int s_qkv = 1, s_o = 1, s_dn = 1;
        {
            TimedScope ts(ctx, SPACE_K_QKV, s);
            if ((rc = run_gemm(ctx, lp.qkv, EPI_F32, ctx->xn, M, ctx->part, hd + 2 * ctx->hd_kv, ctx->part_stride, nullptr, 0,
                               nullptr, s, &s_qkv, nullptr, (ctx->wide_mask & 1) ? ctx->wide_min_rows_qkv : 0, 0)))
                return rc;
        }
        uint16_t* kc_l = (uint16_t*)kv->k + kv_layer * l;
        uint16_t* vc_l = (uint16_t*)kv->v + kv_layer * l;
        // the last layer of a prompt chunk only has to leave its keys and values behind
        const bool kv_only = !out && l + 1 == c.n_layers;
        if (head_attn && !kv_only) {
            HeadAttnLaunch ha{};
            ha.qkv = ctx->part; ha.splits = s_qkv; ha.split_stride = ctx->part_stride;
            ha.cos_t = ctx->cos_t; ha.sin_t = ctx->sin_t; ha.pos = ctx->pos; ha.info = lay.info; ha.kv_len = kv->len;
            ha.kblk = ctx->kblk; ha.vblk = ctx->vblk; ha.kc = kc_l; ha.vc = vc_l;
            ha.batch = B; ha.L = L; ha.Lp = Lp; ha.n_heads = c.n_heads; ha.n_kv_heads = ctx->kv_heads; ha.head_dim = dh;
            ha.capacity = kv->capacity;
            ha.out = ctx->attn_out; ha.out_shape = xs; ha.faults = ctx->faults; ha.paging = paging;
            TimedScope ts(ctx, SPACE_K_ATTN, s);
            HIP_TRY(ctx, launch_head_attention(ha, s));
        } else {
            RopeStore rs{};
            rs.qkv = ctx->part;
            rs.splits = s_qkv;
            rs.split_stride = ctx->part_stride;
            rs.m = M; rs.batch = B; rs.L = L; rs.Lp = Lp; rs.n_heads = c.n_heads; rs.n_kv_heads = ctx->kv_heads; rs.head_dim = dh;
            rs.cos_t = ctx->cos_t; rs.sin_t = ctx->sin_t; rs.pos = ctx->pos; rs.info = lay.info;
            rs.q = ctx->q; rs.q_plane = ctx->q_plane; rs.kblk = ctx->kblk; rs.vblk = ctx->vblk;
            rs.kc = kc_l;
            rs.vc = vc_l;
            rs.capacity = kv->capacity;
            rs.paging = paging;
            rs.faults = ctx->faults;
            // blocks of up to 48 rows: the attention kernel sums, rotates and stores the block itself
            const bool fused_rope = L <= kHeadAttnMaxRows && !kv_only;
            if (!fused_rope) {
                TimedScope ts(ctx, SPACE_K_ROPE, s);
                HIP_TRY(ctx, launch_rope_store(rs, s));
            }
            if (kv_only) break;
            AttnLaunch at{};
            if (fused_rope) {
                at.qkv = ctx->part; at.splits = s_qkv; at.split_stride = ctx->part_stride;
                at.cos_t = ctx->cos_t; at.sin_t = ctx->sin_t; at.pos = ctx->pos;
                at.kc_w = kc_l; at.vc_w = vc_l; at.faults = ctx->faults;
            }
            at.q = ctx->q; at.q_plane = ctx->q_plane; at.kblk = ctx->kblk; at.vblk = ctx->vblk; at.kc = kc_l; at.vc = vc_l;
            at.kv_len = kv->len; at.info = lay.info;
            at.batch = B; at.L = L; at.Lp = Lp; at.n_heads = c.n_heads; at.n_kv_heads = ctx->kv_heads; at.head_dim = dh;
            at.capacity = kv->capacity;
            at.n_wg = attn_wg;
            at.o_part = ctx->o_part; at.ml_part = ctx->ml_part; at.out = ctx->attn_out; at.out_shape = xs; at.paging = paging;
            {
                TimedScope ts(ctx, SPACE_K_ATTN, s);
                HIP_TRY(ctx, launch_attention(at, s));
            }
        }

        {
            TimedScope ts(ctx, SPACE_K_O, s);
            if ((rc = run_gemm(ctx, lp.o, EPI_F32, ctx->attn_out, M, ctx->part, d, ctx->part_stride, nullptr, 0,
                               nullptr, s, &s_o, nullptr, (ctx->wide_mask & 2) ? ctx->wide_min_rows : 0, 1)))
                return rc;
        }
        {
            TimedScope ts(ctx, SPACE_K_NORM, s);
            HIP_TRY(ctx, launch_resid_norm(ctx->x, ctx->part, s_o, ctx->part_stride, d, lp.ffn_norm, c.rms_eps, M, d,
                                           ctx->xn, xs, s));
        }
        {
            TimedScope ts(ctx, SPACE_K_GATE_UP, s);
            if ((rc = run_gemm(ctx, lp.gate_up, EPI_SWIGLU, ctx->xn, M, nullptr, 0, 0, ctx->h, c.ffn, nullptr, s, nullptr, nullptr,
                               (ctx->wide_mask & 4) ? ctx->wide_min_rows : 0, 2)))
                return rc;
        }
        {
            TimedScope ts(ctx, SPACE_K_DOWN, s);
            if ((rc = run_gemm(ctx, lp.down, EPI_F32, ctx->h, M, ctx->part, d, ctx->part_stride, nullptr, 0, nullptr,
                               s, &s_dn, nullptr, (ctx->wide_mask & 8) ? ctx->wide_min_rows : 0, 3)))
                return rc;
        }
        const uint16_t* next_norm = (l + 1 < c.n_layers) ? ctx->layers[l + 1].attn_norm : ctx->final_norm;
        {
            TimedScope ts(ctx, SPACE_K_NORM, s);
            HIP_TRY(ctx, launch_resid_norm(ctx->x, ctx->part, s_dn, ctx->part_stride, d, next_norm, c.rms_eps, M, d,
                                           ctx->xn, xs, s));
        }
    }
    if (!out) {
        ctx->staged_kv = kv->len;
        ctx->staged_groups = G;
        return SPACE_OK;
    }
    int lm_groups = 0;
    {
        TimedScope ts(ctx, SPACE_K_LM_HEAD, s);
        if ((rc = run_gemm(ctx, ctx->lm, EPI_ARGMAX, ctx->xn, M, nullptr, c.vocab, 0, nullptr, 0, out->logits, s, nullptr,
                           &lm_groups, (ctx->wide_mask & 16) ? ctx->wide_min_rows : 0, 4)))
            return rc;
    }

    VerifyLaunch v{};
    v.arg_val = ctx->arg_val; v.arg_idx = ctx->arg_idx; v.arg_groups = ctx->arg_groups;
    v.n_groups_used = lm_groups;
    v.batch = B;
    v.lay = lay;
    if (next_layout) v.next = next_layout->view(); else v.next = LayoutDev{nullptr, nullptr, nullptr, nullptr, 0, 0};
    v.tokens = tokens;
    v.mask_id = c.vocab;
    v.argmax_ws = ctx->argmax_ws; v.argmax = out->argmax;
    v.accepted_len = out->accepted_len; v.accepted_ws = ctx->accepted_ws;
    v.bonus = out->bonus; v.new_cands = out->new_cands; v.max_cands = out->max_cands;
    v.next_tokens = out->next_tokens;
    v.emit = out->emit; v.emit_len = out->emit_len; v.emit_cap = out->emit_cap;
    v.eos_id = out->eos_id; v.finished = out->finished;
    {
        TimedScope ts(ctx, SPACE_K_VERIFY, s);
        HIP_TRY(ctx, launch_verify(v, s));
    }
    ctx->staged_kv = kv->len;
    ctx->staged_groups = G;
    return SPACE_OK;
}

}  // namespace

extern "C" {

int space_step(space_ctx* ctx, const int32_t* tokens, const space_layout* layout, const space_layout* next_layout,
               space_kv* kv, const space_step_out* out, void* stream) {
    if (!ctx) return SPACE_EINVAL;
    if (!tokens || !layout || !out) return fail(ctx, SPACE_EINVAL, "space_step: null argument");
    return step_impl(ctx, tokens, layout, next_layout, kv, out, stream);
}

int space_prefill(space_ctx* ctx, const int32_t* tokens, const space_layout* layout, space_kv* kv, void* stream) {
    if (!ctx) return SPACE_EINVAL;
    if (!tokens || !layout) return fail(ctx, SPACE_EINVAL, "space_prefill: null argument");
    return step_impl(ctx, tokens, layout, nullptr, kv, nullptr, stream);
}

int space_kv_commit(space_ctx* ctx, space_kv* kv, const int32_t* accepted_len, int32_t accepted_all, void* stream) {
    if (!ctx) return SPACE_EINVAL;
    int rc = check_kv(ctx, kv);
    if (rc) return rc;
    if (ctx->staged_kv != kv->len || ctx->staged_groups < 1)
        return fail(ctx, SPACE_EINVAL, "space_kv_commit: no block staged on this cache");
    const int G = ctx->staged_groups;
    if (!accepted_len && (accepted_all < 0 || accepted_all > G - 1))
        return fail(ctx, SPACE_EINVAL, "space_kv_commit: accepted_all %d outside 0..%d", accepted_all, G - 1);
    HIP_TRY(ctx, launch_kv_len_update(kv->len, kv->batch, accepted_len, accepted_all, +1, G - 1, kv->capacity,
                                      (hipStream_t)stream));
    kv->host_len_bound += accepted_len ? G : accepted_all + 1;
    if (kv->host_len_bound > kv->capacity) kv->host_len_bound = kv->capacity;
    ctx->staged_kv = nullptr;
    ctx->staged_groups = 0;
    return SPACE_OK;
}

int space_kv_rollback(space_ctx* ctx, space_kv* kv, const int32_t* n, int32_t n_all, void* stream) {
    if (!ctx) return SPACE_EINVAL;
    int rc = check_kv(ctx, kv);
    if (rc) return rc;
    if (!n && n_all < 0) return fail(ctx, SPACE_EINVAL, "space_kv_rollback: negative count");
    HIP_TRY(ctx, launch_kv_len_update(kv->len, kv->batch, n, n_all, -1, 0, kv->capacity, (hipStream_t)stream));
    if (!n) {
        kv->host_len_bound -= n_all;
        if (kv->host_len_bound < 0) kv->host_len_bound = 0;
    }
    if (ctx->staged_kv == kv->len) {
        ctx->staged_kv = nullptr;
        ctx->staged_groups = 0;
    }
    return SPACE_OK;
}

// Argument checks and launch shared by space_sample_verify and its allocation-free variant; the two
// differ only in where the per-row lists (kept ids, probabilities, counts) and the internal copy of the
// accepted counts live.
static int sample_verify_impl(space_ctx* ctx, const char* who, int32_t batch, const space_layout* layout,
                              const space_layout* next_layout, const space_sample_params* params,
                              const space_sample_io* io, int32_t* row_ids, float* row_probs, int32_t* row_n,
                              int32_t* accepted_ws, size_t rows_max, void* stream) {
    if (!layout || !params || !io) return fail(ctx, SPACE_EINVAL, "%s: null argument", who);
    if (!io->logits || !io->tokens || !io->p_c || !io->uniforms || !io->accepted_len || !io->extra || !io->new_cands ||
        !io->new_pc)
        return fail(ctx, SPACE_EINVAL, "%s: a required buffer is null", who);
    if (params->top_k < 1 || params->top_k > SPACE_MAX_TOP_K)
        return fail(ctx, SPACE_EINVAL, "%s: top_k %d outside 1..%d", who, params->top_k, SPACE_MAX_TOP_K);
    if (!(params->top_p > 0.f) || params->top_p > 1.f)
        return fail(ctx, SPACE_EINVAL, "%s: top_p %g outside (0, 1]", who, (double)params->top_p);
    if (params->residual && (!io->draft_ids || !io->draft_probs))
        return fail(ctx, SPACE_EINVAL, "%s: the residual rule needs draft_ids and draft_probs", who);
    if (layout->L > 16 * kMaxRowTiles)
        return fail(ctx, SPACE_ESHAPE, "%s: blocks of more than %d rows are not verified", who, 16 * kMaxRowTiles);
    if (next_layout && next_layout->L > 16 * kMaxRowTiles)
        return fail(ctx, SPACE_ESHAPE, "%s: next_layout has more than %d rows", who, 16 * kMaxRowTiles);
    if (batch < 1 || (size_t)batch * layout->L > rows_max || batch > ctx->cfg.max_batch)
        return fail(ctx, SPACE_ECAPACITY, "%s: batch %d x %d rows exceeds the limit of %zu rows (max_batch %d)", who,
                    batch, layout->L, rows_max, ctx->cfg.max_batch);
    if (io->max_cands < layout->max_masks || io->max_cands < 1 || io->max_cands > 16 * kMaxRowTiles)
        return fail(ctx, SPACE_EINVAL, "%s: max_cands %d outside %d..%d (the largest mask group .. block limit)", who,
                    io->max_cands, layout->max_masks > 1 ? layout->max_masks : 1, 16 * kMaxRowTiles);
    if (io->next_tokens && !next_layout) return fail(ctx, SPACE_EINVAL, "%s: next_tokens without next_layout", who);
    if (io->emit && (!io->emit_len || io->emit_cap < 1)) return fail(ctx, SPACE_EINVAL, "%s: emit without emit_len/cap", who);
    if (io->eos_id >= 0 && (!io->emit || !io->finished)) return fail(ctx, SPACE_EINVAL, "%s: eos_id needs emit and finished", who);
    SampleLaunch v{};
    v.logits = io->logits; v.vocab = ctx->cfg.vocab; v.batch = batch;
    v.top_k = params->top_k; v.top_p = params->top_p; v.residual = params->residual;
    v.lay = layout->view();
    if (next_layout && io->next_tokens) v.next = next_layout->view();
    v.tokens = io->tokens; v.mask_id = ctx->cfg.vocab;
    v.p_c = io->p_c; v.uniforms = io->uniforms; v.draft_ids = io->draft_ids; v.draft_probs = io->draft_probs;
    v.row_ids = row_ids; v.row_probs = row_probs; v.row_n = row_n;
    v.accepted_len = io->accepted_len; v.accepted_ws = accepted_ws; v.extra = io->extra;
    v.new_cands = io->new_cands; v.new_pc = io->new_pc; v.max_cands = io->max_cands;
    v.new_ids = io->new_ids; v.new_probs = io->new_probs;
    v.next_tokens = v.next.L ? io->next_tokens : nullptr;
    v.emit = io->emit; v.emit_len = io->emit_len; v.emit_cap = io->emit_cap;
    v.eos_id = io->eos_id; v.finished = io->finished;
    v.ratios = io->ratios;
    HIP_TRY(ctx, launch_sample_verify(v, (hipStream_t)stream));
    return SPACE_OK;
}

int space_sample_verify(space_ctx* ctx, int32_t batch, const space_layout* layout, const space_layout* next_layout,
                        const space_sample_params* params, const space_sample_io* io, void* stream) {
    if (!ctx) return SPACE_EINVAL;
    return sample_verify_impl(ctx, "space_sample_verify", batch, layout, next_layout, params, io, ctx->row_ids,
                              ctx->row_probs, ctx->row_n, ctx->accepted_ws, (size_t)ctx->m_max, stream);
}

int space_sample_verify_static(space_ctx* ctx, int32_t batch, const space_layout* layout, const space_layout* next_layout,
                               const space_sample_params* params, const space_sample_io* io, void* stream) {
    if (!ctx) return SPACE_EINVAL;
    if (layout && batch >= 1 && (size_t)batch * layout->L > (size_t)SPACE_STATIC_MAX_ROWS)
        return fail(ctx, SPACE_ECAPACITY, "space_sample_verify_static: batch %d x %d rows exceeds SPACE_STATIC_MAX_ROWS = %d",
                    batch, layout->L, SPACE_STATIC_MAX_ROWS);
    void* base = nullptr;
    HIP_TRY(ctx, static_scratch_address(&base));
    StaticSampleScratch* sc = (StaticSampleScratch*)base;  // a device address: only handed to the kernels
    return sample_verify_impl(ctx, "space_sample_verify_static", batch, layout, next_layout, params, io, sc->row_ids,
                              sc->row_probs, sc->row_n, sc->accepted_ws, (size_t)SPACE_STATIC_MAX_ROWS, stream);
}

int space_sar_loss(space_ctx* ctx, const float* logits, const int32_t* labels, int32_t rows, float* row_loss,
                   float* loss_sum, int32_t* n_terms, void* stream) {
    if (!ctx) return SPACE_EINVAL;
    if (!logits || !labels || !loss_sum || rows < 1) return fail(ctx, SPACE_EINVAL, "space_sar_loss: null argument or no rows");
    if (!row_loss && rows > ctx->m_max)
        return fail(ctx, SPACE_ECAPACITY, "space_sar_loss: %d rows exceed max_batch * max_rows = %d (pass row_loss to lift the limit)",
                    rows, ctx->m_max);
    HIP_TRY(ctx, launch_nll(logits, labels, rows, ctx->cfg.vocab, row_loss ? row_loss : ctx->loss_ws, loss_sum, n_terms,
                            ctx->faults, (hipStream_t)stream));
    return SPACE_OK;
}

int space_sar_transform(const int32_t* tokens, int32_t n_prompt, int32_t n_answer, int32_t k, int32_t mask_id, float p_ar,
                        float u_keep, float u_pos, int32_t* input_ids, int32_t* labels, int32_t* n_input, int32_t* n_labels,
                        int32_t* m_out) {
    if (!tokens || !input_ids || !labels || !n_input || !n_labels || !m_out || n_prompt < 1 || n_answer < 1 || k < 0)
        return SPACE_EINVAL;
    const int n_all = n_prompt + n_answer;
    if (u_keep < p_ar) {  // the sample stays as it is: L_AR
        for (int i = 0; i < n_all; ++i) input_ids[i] = labels[i] = tokens[i];
        *n_input = *n_labels = n_all;
        *m_out = 0;
        return SPACE_OK;
    }
    if (n_answer <= k) return SPACE_ESHAPE;  // no position leaves k + 1 labels
    int m = 1 + (int)std::floor((double)u_pos * (double)(n_answer - k));
    m = std::min(std::max(m, 1), n_answer - k);
    const int kept = n_prompt + m - 1;  // the prompt and y_1 .. y_{m-1}
    for (int i = 0; i < kept; ++i) input_ids[i] = tokens[i];
    for (int j = 0; j < k; ++j) input_ids[kept + j] = mask_id;
    *n_input = kept + k;
    *n_labels = n_prompt + m + k;  // the original tokens through y_{m+k}
    for (int i = 0; i < *n_labels; ++i) labels[i] = tokens[i];
    *m_out = m;
    return SPACE_OK;
}

int space_tune_rows(space_ctx* ctx, int32_t rows, void* stream) {
    if (!ctx) return SPACE_EINVAL;
    if (rows < 1 || rows > ctx->m_max) return fail(ctx, SPACE_ESHAPE, "space_tune_rows: rows outside 1..max_batch*max_rows");
    hipStream_t s = (hipStream_t)stream;
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(s, &cap) != hipSuccess || cap != hipStreamCaptureStatusNone)
        return fail(ctx, SPACE_EINVAL, "space_tune_rows: the stream is being captured (this call measures and waits)");
    const space_config& c = ctx->cfg;
    // the layers whose weights are there take turns, so that no launch finds its weights in a cache
    std::vector<const LayerPacked*> have;
    for (const LayerPacked& l : ctx->layers)
        if (l.qkv.data && l.o.data && l.gate_up.data && l.down.data) have.push_back(&l);
    if (have.empty()) return SPACE_OK;  // weights not handed over yet: nothing to measure on
    size_t turn = 0;
    const int d = c.d_model, hd = ctx->hd;
    const int groups = ceil_div(ceil_div(rows, 16), 2);
    // candidate cuts of `groups` groups of two row tiles into pieces of 4, 3, 2, 1 groups
    std::vector<WideParts> cands;
    auto add = [&](int a, int b, int cc, int dd) {
        if (a < 0 || b < 0 || cc < 0 || dd < 0 || 4 * a + 3 * b + 2 * cc + dd != groups) return;
        for (const WideParts& w : cands)
            if (w.count[0] == a && w.count[1] == b && w.count[2] == cc && w.count[3] == dd) return;
        cands.push_back(WideParts{{a, b, cc, dd}, 1});  // both launch orders
        cands.push_back(WideParts{{a, b, cc, dd}, 0});
    };
    auto rest = [&](int a, int b, int cc, int left) {  // `left` groups as one more piece
        if (left == 3) ++b; else if (left == 2) ++cc; else if (left == 1) return add(a, b, cc, 1);
        add(a, b, cc, 0);
    };
    rest(groups / 4, 0, 0, groups % 4);                                   // pieces of 128 rows: cands[0] is what an unmeasured launch uses
    rest(0, groups / 3, 0, groups % 3);                                   // of 96 rows
    add(0, 0, groups / 2, groups % 2);                                    // of 64 rows
    { const int a = groups / 8; add(a, 0, (groups - 4 * a) / 2, (groups - 4 * a) % 2); }           // half of them large
    { const int a = groups / 4 - 1; if (a >= 0) add(a, 0, (groups - 4 * a) / 2, (groups - 4 * a) % 2); }
    { const int b = groups / 3 - 2; if (b >= 0) add(0, b, (groups - 3 * b) / 2, (groups - 3 * b) % 2); }  // 96 and 64 mixed
    hipEvent_t e0, e1;
    HIP_TRY(ctx, hipEventCreate(&e0));
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return fail(ctx, SPACE_EHIP, "hipEventCreate"); }
    int rc = SPACE_OK;
    for (int cls = 0; cls < 5 && rc == SPACE_OK; ++cls) {
        const int from = !(ctx->wide_mask & (1 << cls)) ? 0 : cls == 0 ? ctx->wide_min_rows_qkv : ctx->wide_min_rows;
        if (from <= 0 || rows < from) continue;
        // The projections whose output is a plain sum also try other numbers of partial sums over the
        // contraction (0: the cost model's).  Whoever reads the partial sums (the attention's staging
        // work, the norm kernels) pays for each of them, which a measurement of the projection alone does
        // not show: the time to read the extra partial sums once is put on top.
        const bool plain = cls == 0 || cls == 1 || cls == 3;
        const int ks_cands[4] = {0, 1, 2, 4};
        float best_ms = 0.f, default_ms = 0.f;
        int best = -1, best_ks = 0;
        for (int kc = 0; kc < (plain ? 4 : 1) && rc == SPACE_OK; ++kc)
        for (int i = 0; i < (int)cands.size() && rc == SPACE_OK; ++i) {
            const int ks = ks_cands[kc];
            if (ks > ctx->part_splits_max) continue;
            float ms_min = 0.f;
            for (int rep = 0; rep < 4 && rc == SPACE_OK; ++rep) {  // the first one warms up
                if (hipEventRecord(e0, s) != hipSuccess) { rc = fail(ctx, SPACE_EHIP, "hipEventRecord"); break; }
                const LayerPacked& lp = *have[turn++ % have.size()];
                switch (cls) {
                    case 0: rc = run_gemm(ctx, lp.qkv, EPI_F32, ctx->xn, rows, ctx->part, hd + 2 * ctx->hd_kv, ctx->part_stride, nullptr, 0, nullptr, s, nullptr, nullptr, 1, -1, &cands[i], ks); break;
                    case 1: rc = run_gemm(ctx, lp.o, EPI_F32, ctx->attn_out, rows, ctx->part, d, ctx->part_stride, nullptr, 0, nullptr, s, nullptr, nullptr, 1, -1, &cands[i], ks); break;
                    case 2: rc = run_gemm(ctx, lp.gate_up, EPI_SWIGLU, ctx->xn, rows, nullptr, 0, 0, ctx->h, c.ffn, nullptr, s, nullptr, nullptr, 1, -1, &cands[i], ks); break;
                    case 3: rc = run_gemm(ctx, lp.down, EPI_F32, ctx->h, rows, ctx->part, d, ctx->part_stride, nullptr, 0, nullptr, s, nullptr, nullptr, 1, -1, &cands[i], ks); break;
                    default: rc = run_gemm(ctx, ctx->lm, EPI_ARGMAX, ctx->xn, rows, nullptr, c.vocab, 0, nullptr, 0, nullptr, s, nullptr, nullptr, 1, -1, &cands[i], ks); break;
                }
                if (rc != SPACE_OK) break;
                float ms = 0.f;
                if (hipEventRecord(e1, s) != hipSuccess || hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess) {
                    rc = fail(ctx, SPACE_EHIP, "space_tune_rows: timing");
                    break;
                }
                if (rep == 1 || (rep > 1 && ms < ms_min)) ms_min = ms;
            }
            if (plain) {  // every partial sum beyond the first is read once more, at about 4 TB/s
                const PackedW& pw = cls == 0 ? have[0]->qkv : cls == 1 ? have[0]->o : have[0]->down;
                const int used = plan_gemm_wide(pw, rows, EPI_F32, ctx->part_splits_max, ks).ksplit;
                const int n_out = cls == 0 ? hd + 2 * ctx->hd_kv : d;
                ms_min += (float)((double)(used - 1) * rows * n_out * 4.0 / 4.0e9);
            }
            if (rc == SPACE_OK && kc == 0 && i == 0) default_ms = ms_min;
            if (rc == SPACE_OK && (best < 0 || ms_min < best_ms)) { best = i; best_ks = ks; best_ms = ms_min; }
        }
        // Same projection back to back is not quite the step's own sequence of kernels: another cut (or
        // split) is taken only where it is clearly ahead.
        if (rc == SPACE_OK && (best > 0 || best_ks > 0) && best_ms < 0.90f * default_ms)
            ctx->wide_parts[((uint64_t)cls << 32) | (uint32_t)rows] = space_ctx::WideTuned{cands[best], best_ks};
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return rc;
}

int space_device_faults(space_ctx* ctx, void* stream) {
    if (!ctx) return SPACE_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    int32_t n = 0;
    HIP_TRY(ctx, hipMemcpyAsync(&n, ctx->faults, sizeof n, hipMemcpyDeviceToHost, s));
    HIP_TRY(ctx, hipStreamSynchronize(s));
    if (n) {
        HIP_TRY(ctx, launch_fill_zero(ctx->faults, 16, s));
        HIP_TRY(ctx, hipStreamSynchronize(s));
    }
    return n;
}

int space_timing_enable(space_ctx* ctx, uint32_t class_mask, int32_t max_records) {
    if (!ctx) return SPACE_EINVAL;
    (void)hipDeviceSynchronize();
    free_events(ctx);
    if (class_mask == 0) return SPACE_OK;
    if (max_records < 1 || class_mask >= (1u << SPACE_K_COUNT))
        return fail(ctx, SPACE_EINVAL, "space_timing_enable: bad mask or record count");
    ctx->ev_start.resize(max_records);
    ctx->ev_stop.resize(max_records);
    ctx->ev_class.assign(max_records, 0);
    for (int i = 0; i < max_records; ++i) {
        ctx->ev_start[i] = nullptr;
        ctx->ev_stop[i] = nullptr;
    }
    for (int i = 0; i < max_records; ++i) {
        if (hipEventCreate(&ctx->ev_start[i]) != hipSuccess || hipEventCreate(&ctx->ev_stop[i]) != hipSuccess) {
            ctx->ev_start.resize(i);
            ctx->ev_stop.resize(i);
            free_events(ctx);
            return fail(ctx, SPACE_EHIP, "hipEventCreate failed");
        }
    }
    // an empty bracket is not free: measure it and take it off every record
    std::vector<float> empty;
    for (int i = 0; i < 9 && i < max_records; ++i) {
        HIP_TRY(ctx, hipEventRecord(ctx->ev_start[i], nullptr));
        HIP_TRY(ctx, hipEventRecord(ctx->ev_stop[i], nullptr));
    }
    HIP_TRY(ctx, hipDeviceSynchronize());
    for (int i = 0; i < 9 && i < max_records; ++i) {
        float ms = 0.f;
        HIP_TRY(ctx, hipEventElapsedTime(&ms, ctx->ev_start[i], ctx->ev_stop[i]));
        empty.push_back(ms);
    }
    std::sort(empty.begin(), empty.end());
    ctx->ev_overhead_ms = empty.empty() ? 0.0 : empty[empty.size() / 2];
    ctx->timing_mask = class_mask;
    return SPACE_OK;
}

int space_timing_read(space_ctx* ctx, void* stream, double* total_ms, int64_t* launches) {
    if (!ctx) return SPACE_EINVAL;
    if (!total_ms || !launches) return fail(ctx, SPACE_EINVAL, "space_timing_read: null argument");
    HIP_TRY(ctx, hipStreamSynchronize((hipStream_t)stream));
    for (int i = 0; i < SPACE_K_COUNT; ++i) {
        total_ms[i] = 0.0;
        launches[i] = 0;
    }
    for (size_t i = 0; i < ctx->ev_used; ++i) {
        float ms = 0.f;
        HIP_TRY(ctx, hipEventElapsedTime(&ms, ctx->ev_start[i], ctx->ev_stop[i]));
        total_ms[ctx->ev_class[i]] += ms > ctx->ev_overhead_ms ? ms - ctx->ev_overhead_ms : 0.0;
        launches[ctx->ev_class[i]] += 1;
    }
    ctx->ev_used = 0;
    return SPACE_OK;
}

int space_debug_buffer(space_ctx* ctx, const char* name, void** ptr, size_t* bytes) {
    if (!ctx) return SPACE_EINVAL;
    if (!name || !ptr || !bytes) return fail(ctx, SPACE_EINVAL, "space_debug_buffer: null argument");
    const space_config& c = ctx->cfg;
    const size_t M = ctx->m_max;
    const std::string n(name);
    const size_t plane_tile = 2 * 64 * 8 * sizeof(uint16_t), rt = ctx->row_tiles_max;
    if (n == "x") { *ptr = ctx->x; *bytes = M * c.d_model * sizeof(float); }
    else if (n == "xn") { *ptr = ctx->xn; *bytes = rt * ctx->kt_d * plane_tile; }
    else if (n == "q") { *ptr = ctx->q; *bytes = 2 * ctx->q_plane * sizeof(uint16_t); }
    else if (n == "attn_out") { *ptr = ctx->attn_out; *bytes = rt * ctx->kt_hd * plane_tile; }
    else if (n == "h") { *ptr = ctx->h; *bytes = rt * ctx->kt_ffn * plane_tile; }
    else if (n == "pos") { *ptr = ctx->pos; *bytes = M * sizeof(int32_t); }
    else return fail(ctx, SPACE_EINVAL, "space_debug_buffer: unknown buffer '%s'", name);
    return SPACE_OK;
}

}  // extern "C"
