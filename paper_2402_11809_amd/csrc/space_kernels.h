// Internal launch interface between the C ABI (space_api.hip) and the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace space {

constexpr int kTileN = 16;        // weight rows per MFMA tile
constexpr int kTileK = 32;        // contraction elements per MFMA tile
constexpr int kTileBytes = 1024;  // one packed 16x32 bf16 tile
constexpr int kMaxRowTiles = 6;   // 96 rows per projection pass; also the longest block the verification handles
constexpr int kMaxBlockRows = 1024;  // longest block of one sequence (prompt chunks; no verification beyond 96 rows)
constexpr int kAttnKeys = 32;     // keys per attention chunk; V is stored transposed in runs of 32

inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
inline int round_up(int a, int b) { return ceil_div(a, b) * b; }

enum GemmEpilogue { EPI_F32 = 0, EPI_SWIGLU = 1, EPI_ARGMAX = 2 };

// Shape of an activation matrix X[rows, k] in operand ("tile") order.  Contraction tile kt holds,
// for every row tile t, a hi plane and a lo plane; a full plane is 64 lanes x 8 elements (1 KB,
// lane l = row t*16 + l%16, columns kt*32 + 8*(l/16)..+8).  The last row tile stores only its
// last_cols = rows - 16*(row_tiles - 1) real rows, as [4 column groups][last_cols][8]: a block of
// 36 rows then costs 2.25 tiles of traffic per workgroup and contraction tile instead of 3.
struct XtShape {
    int row_tiles;
    int last_cols;  // 1 .. 16
};
inline XtShape xt_shape(int rows) {
    XtShape x;
    x.row_tiles = ceil_div(rows, 16);
    x.last_cols = rows - 16 * (x.row_tiles - 1);
    return x;
}

// Packed weight matrix.  Tiles of 16 rows x 32 columns (1 KB, lane l owns bytes [16 l, 16 l + 16) =
// row l%16, columns 8*(l/16)..+8 of the tile) are stored in the order the projection kernel streams
// them: the contraction is cut into 4 * splits equal ranges of lq tiles (one per wave of a
// workgroup and per split), rows into groups of r_pack tiles, and tile (nt, kt) lives at KB index
//   ((i * (splits * groups * 4) + ((s * groups + g) * 4 + w)) * r_pack + r)
// with g = nt / r_pack, r = nt % r_pack, s * 4 + w = kt / lq, i = kt % lq.  At loop iteration i the
// whole grid therefore reads one contiguous window, which is what the HBM controllers like best.
// Rows / columns beyond n / k (up to groups * r_pack tiles and 4 * splits * lq tiles) are zero.
struct PackedW {
    const void* data = nullptr;
    int n = 0, k = 0;          // logical rows / columns
    int n_tiles = 0, k_tiles = 0;
    int r_pack = 4;            // tiles per row group (2, 4, 6 or 8)
    int splits = 1;            // partial results over the contraction
    int lq = 0;                // contraction tiles per wave
    int groups = 0;            // row groups
    int k_tiles_pad() const { return 4 * splits * lq; }
    size_t bytes() const { return (size_t)lq * splits * groups * 4 * r_pack * kTileBytes; }
};

struct GemmLaunch {
    PackedW w;
    const uint16_t* x;  // activation planes in tile order (XtShape)
    XtShape xs;         // shape of the whole activation matrix
    int row_tile0;      // first row tile this launch covers
    int m;              // rows of this launch, starting at row_tile0 * 16: 1 .. 96, or up to 96 * passes
    int passes;         // 1, or the number of 96-row passes that share this launch (then row_tile0 == 0)
    int tiles_per_wave; // weight tiles per wave, gemm_tiles_per_wave(w, rows of the whole matrix)
    // EPI_F32: out[s][m][ldo] fp32 partial sums
    float* out;
    int ldo;
    size_t split_stride;  // elements between partials
    // EPI_SWIGLU: weight tiles alternate gate / up; h = silu(gate) * up as operand planes of shape xs
    uint16_t* h;
    int ffn;
    // EPI_ARGMAX: logits (nullable) [m, ldo]; per row and workgroup the (max, lowest index) pair
    float* arg_val;
    int32_t* arg_idx;
    int arg_groups;  // row stride of arg_val / arg_idx
};

// Packs up to three row-major bf16 matrices with k columns each into w->data (w->bytes() bytes).
// interleave == 0: rows are concatenated (s0 rows, then s1, then s2).  interleave == 1 (gate / up):
// even tiles take 16 rows of s0, odd tiles the same 16 rows of s1.
hipError_t launch_pack(const void* s0, int n0, const void* s1, int n1, const void* s2, int n2, int interleave,
                       const PackedW& w, void* dst, hipStream_t s);
void plan_packed(PackedW* w, int n, int k, int r_pack, int splits);
hipError_t launch_gemm(const GemmLaunch& g, GemmEpilogue epi, hipStream_t s);
int gemm_tiles_per_wave(const PackedW& w, int total_rows);
int gemm_groups(const PackedW& w, int tiles_per_wave);  // workgroups along the rows of W

// The same projections for many rows (prompt chunks, batches of blocks), where the matrix unit and not
// the weight stream is the limit: workgroups of 8 waves x tiles_per_wave weight tiles x 128 rows with
// the activation planes shared through LDS.  Reads the same packed matrices.  The plan picks, for
// EPI_F32, a split of the contraction into ksplit partial sums out[s] (at most max_splits; the caller
// adds them up as it does the skinny kernel's).
constexpr int kWideRowTiles = 8;  // at most 128 rows per workgroup
// How the rows of every weight group are cut: count[c] pieces of 4 - c groups of two row tiles (8, 6, 4,
// 2 row tiles), laid end to end in this order; the groups add up to ceil(ceil(m / 16) / 2).
struct WideParts {
    int count[4];
    int by_size;  // launch order: 0 = weight group by weight group, 1 = all pieces of a size before any smaller one
};
struct WidePlan {
    WideParts parts;
    int tiles_per_wave;  // 2
    int n_groups;        // workgroups along the rows of W (EPI_ARGMAX: partials per row)
    int ksplit;          // partial sums over the contraction
    int kt_per_split;    // contraction tiles per partial sum
};
// force_ksplit > 0: that many partial sums over the contraction instead of the cost model's choice
// (plain-sum epilogue only; rounded down to what leaves every split at least one pipeline round)
WidePlan plan_gemm_wide(const PackedW& w, int m, GemmEpilogue epi, int max_splits, int force_ksplit = 0);
// g.passes and g.tiles_per_wave are ignored (the plan's pieces are used); g.row_tile0 must be 0.
hipError_t launch_gemm_wide(const GemmLaunch& g, const WidePlan& p, GemmEpilogue epi, hipStream_t s);

struct LayoutDev {
    const int32_t* info;     // [L] (group << 1) | is_mask
    const int32_t* rel_pos;  // [L]
    const int32_t* real_row; // [G] row of the non-mask token of each group
    const int32_t* n_mask;   // [G]
    int L, G;
};

// cos / sin of every position 0 .. n_pos-1 ([n_pos][head_dim/2] each), computed once
hipError_t launch_rope_table(float* cos_t, float* sin_t, int n_pos, int head_dim, float rope_base, hipStream_t s);
// Embedding rows -> x, position ids, the rows' rotary factors (copied out of the table; positions outside it are
// clamped) and the first RMSNorm: xn = operand planes of x * rsqrt(mean(x^2) + eps) * norm_w.
hipError_t launch_embed(const int32_t* tokens, const uint16_t* embed, int vocab, int d, const LayoutDev& lay,
                        const int32_t* kv_len, int batch, const float* cos_tab, const float* sin_tab, int n_pos,
                        int head_dim, float* x, int32_t* pos, float* cos_t, float* sin_t, int32_t* faults,
                        const uint16_t* norm_w, float eps, uint16_t* xn, XtShape xs, hipStream_t s);

// x += sum_s part[s]; xn = operand planes of x * rsqrt(mean(x^2) + eps) * w
hipError_t launch_resid_norm(float* x, const float* part, int splits, size_t split_stride, int ldp,
                             const uint16_t* w, float eps, int m, int d, uint16_t* xn, XtShape xs, hipStream_t s);

// Where the cache keeps the 32-position run `chunk` of (sequence b, key/value head kvh), in elements
// from the layer's base: contiguous caches [B][Hkv][capacity][dh], or pages [n_pages][Hkv][32][dh]
// looked up in table[b * table_stride + chunk] (entries clamped to the pool).  K and V runs have the
// same size and order of runs, so one offset serves both.
struct KvPaging {
    const int32_t* table = nullptr;  // nullptr: contiguous
    int table_stride = 0;
    int n_pages = 0;
};

struct RopeStore {
    const float* qkv;  // [splits][m][(n_heads + 2 n_kv_heads) * head_dim]: q heads, then k heads, then v heads
    int splits;
    size_t split_stride;
    int m, batch, L, Lp, n_heads, n_kv_heads, head_dim;
    const float* cos_t;
    const float* sin_t;
    const int32_t* pos;
    const int32_t* info;
    uint16_t* q;     // [hi, lo][B][H][L][dh]
    size_t q_plane;  // elements between the hi and the lo plane
    uint16_t* kblk;  // [B][Hkv][Lp][dh]
    uint16_t* vblk;  // [B][Hkv][Lp/32][dh][32]
    uint16_t* kc;    // cache of this layer [B][Hkv][cap][dh]
    uint16_t* vc;    // cache of this layer [B][Hkv][cap/32][dh][32]
    int capacity;
    KvPaging paging;
    int32_t* faults;
};
hipError_t launch_rope_store(const RopeStore& a, hipStream_t s);

constexpr int kHeadAttnMaxRows = 48;  // longest block the fused rotary + attention kernels take
struct AttnLaunch {
    const uint16_t* q;
    size_t q_plane;
    const uint16_t* kblk;
    const uint16_t* vblk;
    const uint16_t* kc;
    const uint16_t* vc;
    const int32_t* kv_len;
    const int32_t* info;
    int batch, L, Lp, n_heads, n_kv_heads, head_dim, capacity;
    int n_wg;        // workgroups along the key axis: attention_workgroups(upper bound of len, L, streams)
    float* o_part;   // [B][H][n_wg][L][dh]
    float* ml_part;  // [B][H][n_wg][L][2]
    uint16_t* out;   // operand planes of the attention output, [B*L rows, n_heads*head_dim]
    XtShape out_shape;
    KvPaging paging;
    // Blocks of at most kHeadAttnMaxRows rows can skip the rotary / store launch in front: with qkv set
    // (the QKV projection's partial sums, as in HeadAttnLaunch) every workgroup sums and rotates the
    // block's queries itself and the last workgroup along the keys does the same for the block's keys
    // and values, keeps them in LDS, writes the non-mask rows to their cache slots (kc_w / vc_w: the
    // same memory as kc / vc) and takes the block's own chunks.  q, kblk and vblk are then unused.
    const float* qkv = nullptr;
    int splits = 0;
    size_t split_stride = 0;
    const float* cos_t = nullptr;
    const float* sin_t = nullptr;
    const int32_t* pos = nullptr;
    uint16_t* kc_w = nullptr;
    uint16_t* vc_w = nullptr;
    int32_t* faults = nullptr;
};
hipError_t launch_attention(const AttnLaunch& a, hipStream_t s);
int attention_workgroups(int len_bound, int L, int streams);

// Rotary, K/V store, attention and normalisation of a block of at most kHeadAttnMaxRows rows in one
// launch, one workgroup per (sequence, head, tile of 16 query rows).  Reads the QKV projection's
// split partials; writes one staging slice per workgroup, the cache slots of the non-mask rows
// and the output's operand planes.
struct HeadAttnLaunch {
    const float* qkv;  // [splits][batch * L][(n_heads + 2 n_kv_heads) * head_dim]
    int splits;
    size_t split_stride;
    const float* cos_t;
    const float* sin_t;
    const int32_t* pos;
    const int32_t* info;
    const int32_t* kv_len;
    uint16_t* kblk;  // [B][H][query tiles][Lp][dh]
    uint16_t* vblk;  // [B][H][query tiles][Lp/32][dh][32]
    uint16_t* kc;    // cache of this layer, [B][n_kv_heads][...]
    uint16_t* vc;
    int batch, L, Lp, n_heads, n_kv_heads, head_dim, capacity;
    uint16_t* out;  // operand planes, [B*L rows, n_heads*head_dim]
    XtShape out_shape;
    KvPaging paging;
    int32_t* faults;
};
hipError_t launch_head_attention(const HeadAttnLaunch& a, hipStream_t s);

struct VerifyLaunch {
    const float* arg_val;
    const int32_t* arg_idx;
    int arg_groups, n_groups_used;
    int batch;
    LayoutDev lay;
    LayoutDev next;  // next.L == 0: no next block
    const int32_t* tokens;
    int mask_id;
    int32_t* argmax_ws;  // [B*L] internal
    int32_t* argmax;     // nullable outputs ...
    int32_t* accepted_len;
    int32_t* accepted_ws;  // [B] internal copy
    int32_t* bonus;
    int32_t* new_cands;
    int max_cands;
    int32_t* next_tokens;
    int32_t* emit;
    int32_t* emit_len;
    int emit_cap;
    int eos_id;          // < 0: none
    int32_t* finished;   // [B], sticky
};
hipError_t launch_verify(const VerifyLaunch& v, hipStream_t s);

// Rejection-sampling verification (Algorithm 1 as printed): warped distribution of every block row,
// then the acceptance loop, the extra token and the candidate refresh.
constexpr int kMaxTopK = 64;
struct SampleLaunch {
    const float* logits;  // [B][L][vocab]
    int vocab, batch;
    int top_k;
    float top_p;
    int residual;
    LayoutDev lay;
    LayoutDev next;       // next.L == 0: no next block
    const int32_t* tokens;
    int mask_id;
    const float* p_c;
    const float* uniforms;
    const int32_t* draft_ids;
    const float* draft_probs;
    // scratch: kept ids / probabilities / count of every row
    int32_t* row_ids;     // [B*L][kMaxTopK]
    float* row_probs;     // [B*L][kMaxTopK]
    int32_t* row_n;       // [B*L]
    int32_t* accepted_len;
    int32_t* accepted_ws;
    int32_t* extra;
    int32_t* new_cands;
    float* new_pc;
    int max_cands;
    int32_t* new_ids;
    float* new_probs;
    int32_t* next_tokens;
    int32_t* emit;
    int32_t* emit_len;
    int emit_cap;
    float* ratios;
    int eos_id;          // < 0: none
    int32_t* finished;   // [B], sticky
};
hipError_t launch_sample_verify(const SampleLaunch& v, hipStream_t s);

// row_loss[r] = -log softmax(logits[r])[labels[r]] (0 for labels < 0), then loss_sum = their sum in row
// order and n_terms = the number of rows that count.
hipError_t launch_nll(const float* logits, const int32_t* labels, int rows, int vocab, float* row_loss, float* loss_sum,
                      int32_t* n_terms, int32_t* faults, hipStream_t s);

hipError_t launch_kv_len_update(int32_t* len, int batch, const int32_t* delta_dev, int delta_all, int sign,
                                int clamp_hi, int capacity, hipStream_t s);
hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t s);

}  // namespace space
