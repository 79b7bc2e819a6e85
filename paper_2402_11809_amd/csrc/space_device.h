// Device-side helpers shared by the kernel sources: operand types, bf16 splitting, the activation
// ("tile order") and packed-weight index maps, and the MFMA wrapper.
#pragma once
#include "space_kernels.h"

namespace space {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;

__device__ __forceinline__ uint16_t f2bf(float f) {  // round to nearest even (v_cvt_pk_bf16_f32)
    return __builtin_bit_cast(uint16_t, (__bf16)f);
}
__device__ __forceinline__ float bf2f(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
// Activations feed the matrix unit as two bf16 planes, hi = bf16(x) and lo = bf16(x - hi), so that
// the product keeps about 16 mantissa bits of x; the weights (and the K/V cache) are exact bf16.
// Operand layout of an activation matrix ("tile order"): see XtShape.  A wave reads a full plane
// with one contiguous 1-KB load and the ragged last row tile with a 64 * last_cols byte one.
__device__ __forceinline__ size_t xt_index(int m, int k, XtShape xs, int plane) {
    const int kt = k >> 5, t = m >> 4, kc = (k & 31) >> 3;
    const int c = (t == xs.row_tiles - 1) ? xs.last_cols : 16;
    const size_t kstride = (size_t)(xs.row_tiles - 1) * 1024 + 64 * xs.last_cols;
    return kt * kstride + (size_t)t * 1024 + (plane * 4 + kc) * c * 8 + (m & 15) * 8 + (k & 7);
}
__device__ __forceinline__ void xt_store(uint16_t* xt, int m, int k, XtShape xs, float v) {
    const uint16_t hi = f2bf(v);
    xt[xt_index(m, k, xs, 0)] = hi;
    xt[xt_index(m, k, xs, 1)] = f2bf(v - bf2f(hi));
}
__device__ __forceinline__ f32x4 mfma16(u32x4 a, u32x4 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c,
                                                   0, 0, 0);
}

// Maximum / sum over the four lanes l, l ^ 16, l ^ 32, l ^ 48 (one row of an MFMA result tile lives in
// these), returned in all four.  gfx950's row-swap instructions do it inside the vector ALU: with both
// operands equal, v_permlane16_swap returns (rows 0 0 2 2, rows 1 1 3 3) and v_permlane32_swap (lower
// half twice, upper half twice), so two swaps and two operations replace two trips through the LDS
// crossbar.
__device__ __forceinline__ float row_groups_max(float v) {
    // (the two halves of a result are copied to scalars before their bits are reinterpreted: a bit cast
    // applied to a vector element directly reads element 0 with this compiler)
    const unsigned vb = __builtin_bit_cast(unsigned, v);
    const u32x2 s = __builtin_amdgcn_permlane16_swap(vb, vb, false, false);
    const unsigned s0 = s[0], s1 = s[1];
    const float m = fmaxf(__builtin_bit_cast(float, s0), __builtin_bit_cast(float, s1));
    const unsigned mb = __builtin_bit_cast(unsigned, m);
    const u32x2 r = __builtin_amdgcn_permlane32_swap(mb, mb, false, false);
    const unsigned r0 = r[0], r1 = r[1];
    return fmaxf(__builtin_bit_cast(float, r0), __builtin_bit_cast(float, r1));
}
__device__ __forceinline__ float row_groups_sum(float v) {
    const unsigned vb = __builtin_bit_cast(unsigned, v);
    const u32x2 s = __builtin_amdgcn_permlane16_swap(vb, vb, false, false);
    const unsigned s0 = s[0], s1 = s[1];
    const float m = __builtin_bit_cast(float, s0) + __builtin_bit_cast(float, s1);
    const unsigned mb = __builtin_bit_cast(unsigned, m);
    const u32x2 r = __builtin_amdgcn_permlane32_swap(mb, mb, false, false);
    const unsigned r0 = r[0], r1 = r[1];
    return __builtin_bit_cast(float, r0) + __builtin_bit_cast(float, r1);
}

__device__ __forceinline__ size_t packed_tile_index(const PackedW& w, int nt, int kt) {
    const int g = nt / w.r_pack, r = nt % w.r_pack;
    const int q = kt / w.lq, i = kt % w.lq;
    const int s = q >> 2, wv = q & 3;
    return ((size_t)i * ((size_t)w.splits * w.groups * 4) + ((size_t)s * w.groups + g) * 4 + wv) * w.r_pack + r;
}

// Element offset, from the layer's cache base, of the 32-position run `chunk` of (sequence b, key/value
// head kvh); see KvPaging.  *bad is set when a table entry lies outside the pool (the entry is clamped).
template <bool PAGED>
__device__ __forceinline__ size_t kv_run_offset(const KvPaging& pg, int b, int kvh, int n_kv_heads, int capacity,
                                                int dh, int chunk, bool* bad = nullptr) {
    if (!PAGED) return (((size_t)b * n_kv_heads + kvh) * capacity + (size_t)chunk * kAttnKeys) * dh;
    int page = pg.table[(size_t)b * pg.table_stride + chunk];
    if (page < 0 || page >= pg.n_pages) {
        if (bad) *bad = true;
        page = min(max(page, 0), pg.n_pages - 1);
    }
    return ((size_t)page * n_kv_heads + kvh) * kAttnKeys * dh;
}

}  // namespace space
