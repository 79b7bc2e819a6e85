// Internal launch interface between the C ABI (space_api.hip) and the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace space {

constexpr int kTileN = 16;        // weight rows per MFMA tile
constexpr int kTileK = 32;        // contraction elements per MFMA tile
constexpr int kTileBytes = 1024;  // one packed 16x32 bf16 tile
constexpr int kMaxRowTiles = 6;   // 96 rows per projection pass
constexpr int kAttnKeys = 32;     // keys per attention chunk; V is stored transposed in runs of 32

inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
inline int round_up(int a, int b) { return ceil_div(a, b) * b; }

enum GemmEpilogue { EPI_F32 = 0, EPI_SWIGLU = 1, EPI_ARGMAX = 2 };

// Packed weight matrix: tiles of 16 rows x 32 columns, tile (nt, kt) at ((nt * k_tiles) + kt) KB,
// lane l of a wave owns bytes [16 l, 16 l + 16) = row nt*16 + l%16, columns kt*32 + 8*(l/16) .. +8.
struct PackedW {
    const void* data = nullptr;
    int n = 0, k = 0;          // logical rows / columns
    int n_tiles = 0, k_tiles = 0;
};

struct GemmLaunch {
    PackedW w;
    const uint16_t* x;  // activation planes in tile order, [k_tiles][row_tiles][hi, lo][64 lanes][8]
    int row_tiles;      // row tiles of the whole activation matrix
    int row_tile0;      // first row tile this launch covers
    int m;              // rows of this launch, 1 .. 96, starting at row_tile0 * 16
    int tiles_per_wave; // weight tiles per wave: 4 (at most 48 rows) or 2
    int splits;         // partial results over the contraction (1 for SWIGLU / ARGMAX)
    // EPI_F32: out[s][m][ldo] fp32 partial sums
    float* out;
    int ldo;
    size_t split_stride;  // elements between partials
    // EPI_SWIGLU: weight tiles alternate gate / up; h = silu(gate) * up as operand planes (row_tiles rows)
    uint16_t* h;
    int ffn;
    // EPI_ARGMAX: logits (nullable) [m, ldo]; per row and workgroup the (max, lowest index) pair
    float* arg_val;
    int32_t* arg_idx;
    int arg_groups;  // row stride of arg_val / arg_idx
};

// Packs up to three row-major bf16 matrices with k columns each.  interleave == 0: rows are
// concatenated (s0 rows, then s1, then s2).  interleave == 1 (gate / up): even tiles take 16 rows of
// s0, odd tiles the same 16 rows of s1.  Rows / columns past the sources are zero.
hipError_t launch_pack(const void* s0, int n0, const void* s1, int n1, const void* s2, int n2, int interleave,
                       int k, void* dst, int n_tiles, int k_tiles, hipStream_t s);
hipError_t launch_gemm(const GemmLaunch& g, GemmEpilogue epi, hipStream_t s);
int gemm_tiles_per_wave(int total_rows);  // 4 while the accumulators of 3 row tiles fit, else 2
int gemm_groups(const PackedW& w, int tiles_per_wave);

struct LayoutDev {
    const int32_t* info;     // [L] (group << 1) | is_mask
    const int32_t* rel_pos;  // [L]
    const int32_t* real_row; // [G] row of the non-mask token of each group
    const int32_t* n_mask;   // [G]
    int L, G;
};

hipError_t launch_embed(const int32_t* tokens, const uint16_t* embed, int vocab, int d, const LayoutDev& lay,
                        const int32_t* kv_len, int batch, float rope_base, int head_dim, float* x, int32_t* pos,
                        float* cos_t, float* sin_t, int32_t* faults, hipStream_t s);

// x += sum_s part[s]; xn = operand planes of x * rsqrt(mean(x^2) + eps) * w
hipError_t launch_resid_norm(float* x, const float* part, int splits, size_t split_stride, int ldp,
                             const uint16_t* w, float eps, int m, int d, uint16_t* xn, int row_tiles, hipStream_t s);

struct RopeStore {
    const float* qkv;  // [splits][m][3*hd]
    int splits;
    size_t split_stride;
    int m, batch, L, Lp, n_heads, head_dim;
    const float* cos_t;
    const float* sin_t;
    const int32_t* pos;
    const int32_t* info;
    uint16_t* q;     // [hi, lo][B][H][L][dh]
    size_t q_plane;  // elements between the hi and the lo plane
    uint16_t* kblk;  // [B][H][Lp][dh]
    uint16_t* vblk;  // [B][H][Lp/32][dh][32]
    uint16_t* kc;    // cache of this layer [B][H][cap][dh]
    uint16_t* vc;    // cache of this layer [B][H][cap/32][dh][32]
    int capacity;
    int32_t* faults;
};
hipError_t launch_rope_store(const RopeStore& a, hipStream_t s);

struct AttnLaunch {
    const uint16_t* q;
    size_t q_plane;
    const uint16_t* kblk;
    const uint16_t* vblk;
    const uint16_t* kc;
    const uint16_t* vc;
    const int32_t* kv_len;
    const int32_t* info;
    int batch, L, Lp, n_heads, head_dim, capacity, n_splits;
    float* o_part;   // [B][H][n_splits+1][L][dh]
    float* ml_part;  // [B][H][n_splits+1][L][2]
    uint16_t* out;   // operand planes of the attention output, [B*L rows, n_heads*head_dim]
    int out_row_tiles;
};
hipError_t launch_attention(const AttnLaunch& a, hipStream_t s);

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
};
hipError_t launch_verify(const VerifyLaunch& v, hipStream_t s);

hipError_t launch_kv_len_update(int32_t* len, int batch, const int32_t* delta_dev, int delta_all, int sign,
                                int clamp_hi, int capacity, hipStream_t s);
hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t s);

}  // namespace space
