// gfx950 kernels of the SPACE auto-correct decoding step (arxiv 2402.11809, Algorithm 1).
//
// One model invocation over the step block is memory bound on the weight stream (the paper's
// premise: decoding is bounded by memory bandwidth, so the extra k(k+2) rows ride for free).
// Hence: weights are pre-packed into MFMA operand order and streamed once with 16-byte
// non-temporal loads; the few activation rows are the other MFMA operand; all small
// per-row work (residual add, RMSNorm, rotary, SwiGLU, argmax) is fused into the kernels
// that already touch the data.
//
// MFMA used throughout: v_mfma_f32_16x16x32_bf16, D[16x16] += A[16x32] * B[32x16].
//   A: lane l holds row l%16,  contraction slots (l/16, j), j = 0..7
//   B: lane l holds col l%16,  contraction slots (l/16, j)
//   D: lane l holds col l%16,  rows 4*(l/16) + i, i = 0..3
// The contraction is order independent, so any assignment of slots to real indices is fine as
// long as A and B agree.
#include "space_kernels.h"
#include "space_device.h"

#include <limits.h>
#include <type_traits>
#include <math.h>
#include <stdlib.h>
#include <string.h>

namespace space {

// ------------------------------------------------------------------------------------------
// fill / weight packing (init time)
// ------------------------------------------------------------------------------------------

__global__ void fill_zero_kernel(u32x4* p, size_t n16, uint8_t* tail, size_t ntail) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    const u32x4 z = {0, 0, 0, 0};
    for (; i < n16; i += stride) p[i] = z;
    if (blockIdx.x == 0 && threadIdx.x < ntail) tail[threadIdx.x] = 0;
}

hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t s) {
    if (bytes == 0) return hipSuccess;
    const size_t n16 = bytes / 16, ntail = bytes % 16;
    size_t blocks = (n16 + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    if (blocks == 0) blocks = 1;
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)blocks), dim3(256), 0, s, (u32x4*)p, n16,
                       (uint8_t*)p + n16 * 16, ntail);
    return hipGetLastError();
}

__global__ __launch_bounds__(64) void pack_kernel(const uint16_t* s0, int n0, const uint16_t* s1, int n1,
                                                  const uint16_t* s2, int n2, int interleave, PackedW w, u32x4* dst) {
    const int lane = threadIdx.x;
    const int kt = blockIdx.x, nt = blockIdx.y;
    const int rl = lane & 15, kc = lane >> 4;
    const int k = w.k;
    const uint16_t* src = nullptr;
    int row = -1;
    if (interleave) {
        row = (nt >> 1) * 16 + rl;
        src = (nt & 1) ? s1 : s0;
        if (row >= n0) src = nullptr;
    } else {
        int R = nt * 16 + rl;
        if (R < n0) { src = s0; row = R; }
        else if (R < n0 + n1) { src = s1; row = R - n0; }
        else if (R < n0 + n1 + n2) { src = s2; row = R - n0 - n1; }
    }
    uint32_t v4[4] = {0, 0, 0, 0};
    if (src) {
        for (int j = 0; j < 8; ++j) {
            const int col = kt * 32 + kc * 8 + j;
            const uint32_t v = (col < k) ? src[(size_t)row * k + col] : 0u;
            v4[j >> 1] |= v << (16 * (j & 1));
        }
    }
    u32x4 o = {v4[0], v4[1], v4[2], v4[3]};
    dst[packed_tile_index(w, nt, kt) * 64 + lane] = o;
}

void plan_packed(PackedW* w, int n, int k, int r_pack, int splits) {
    w->n = n;
    w->k = k;
    w->n_tiles = ceil_div(n, kTileN);
    w->k_tiles = ceil_div(k, kTileK);
    w->r_pack = r_pack;
    w->splits = splits;
    w->lq = ceil_div(w->k_tiles, 4 * splits);
    w->groups = ceil_div(w->n_tiles, r_pack);
}

hipError_t launch_pack(const void* s0, int n0, const void* s1, int n1, const void* s2, int n2, int interleave,
                       const PackedW& w, void* dst, hipStream_t s) {
    hipLaunchKernelGGL(pack_kernel, dim3(w.k_tiles_pad(), w.groups * w.r_pack), dim3(64), 0, s, (const uint16_t*)s0,
                       n0, (const uint16_t*)s1, n1, (const uint16_t*)s2, n2, interleave, w, (u32x4*)dst);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// skinny projection: out[m, n] = sum_k x[m, k] * W[n, k], m <= 96, weights streamed once
// ------------------------------------------------------------------------------------------
//
// grid = (weight-tile groups of R tiles, splits of the contraction); 4 waves per workgroup share
// the R weight tiles and each take a quarter of the workgroup's contraction range, then add
// their accumulators through LDS in a fixed order (results are reproducible bit for bit).
// Per contraction tile a wave issues R 1-KB weight loads (HBM, each one contiguous), 2T 1-KB
// activation loads (hi and lo plane, L2 resident) and 2*R*T MFMAs; D tiles are kept in flight
// per wave.

// Weight tiles are read once per launch when the block fits one pass (up to 3 row tiles here): then a
// non-temporal load keeps them from displacing the activation planes in L2.  The variants for more
// row tiles may run several passes per launch and want the tiles kept for the sibling passes.
template <int T>
__device__ __forceinline__ u32x4 load_weight_tile(const u32x4* p) {
    if (T <= 3) return __builtin_nontemporal_load(p);
    return *p;
}

template <int T, int R, int EPI, int D>
__global__ __launch_bounds__(256) void gemm_skinny_kernel(GemmLaunch g) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int bx = blockIdx.x, s = blockIdx.y, pass = 0;
    if (T >= 4 && g.passes > 1) {
        // More than 16*T rows: every (weight group, split) runs once per pass of 16*T rows, all in one
        // launch.  Workgroup index -> XCD is index % 8, so the passes of one weight group get indices
        // that differ by 8: they run on the same XCD at about the same time and the weight tiles
        // cross HBM once (ordinary loads below, so that L2 keeps them for the sibling passes).
        const int q = blockIdx.x >> 3, n_gs = (g.w.groups * g.w.r_pack / R) * g.w.splits;
        pass = q % g.passes;
        const int gi = (q / g.passes) * 8 + (blockIdx.x & 7);
        if (gi >= n_gs) return;
        bx = gi % (n_gs / g.w.splits);
        s = gi / (n_gs / g.w.splits);
    }
    const int nt0 = bx * R;
    const int row_tile0 = g.row_tile0 + pass * T;
    const int m_rows = T >= 4 ? min(g.m - pass * 16 * T, 16 * T) : g.m;  // rows of this pass
    const int t_run = T >= 4 ? (m_rows + 15) >> 4 : T;                    // its row tiles, 1 .. T
    // this wave's contraction range: lq tiles starting at (s * 4 + wave) * lq (tiles past k_tiles are zero)
    const int kw0 = (s * 4 + wave) * g.w.lq, kw1 = kw0 + g.w.lq;
    const size_t wstep = (size_t)g.w.splits * g.w.groups * 4 * g.w.r_pack * 64;  // u32x4 per loop iteration
    const u32x4* wp[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int nt = nt0 + r;  // always inside the padded tile grid
        const size_t first = (((size_t)s * g.w.groups + nt / g.w.r_pack) * 4 + wave) * g.w.r_pack + nt % g.w.r_pack;
        wp[r] = (const u32x4*)g.w.data + first * 64 + lane;
    }
    // Activation planes of this pass's row tile t at contraction tile kt, in 16-byte units:
    // kt * xkt + t * 128 + (lane | 64 + lane), except for the ragged last tile of the matrix, where the
    // lanes of columns past last_cols re-read column last_cols - 1 (their results are never stored).
    // Tiles past the end of a short last pass repeat its last real tile.
    const u32x4* xp = (const u32x4*)g.x + (size_t)row_tile0 * 128;
    const size_t xkt = (size_t)(g.xs.row_tiles - 1) * 128 + 8 * g.xs.last_cols;
    int boff[2 * T];
#pragma unroll
    for (int t = 0; t < T; ++t) {
        const int tt = min(t, t_run - 1);
        const int c = (row_tile0 + tt == g.xs.row_tiles - 1) ? g.xs.last_cols : 16;
        boff[2 * t] = tt * 128 + (lane >> 4) * c + min(lane & 15, c - 1);
        boff[2 * t + 1] = boff[2 * t] + 4 * c;
    }

    f32x4 acc[R][T];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int t = 0; t < T; ++t) acc[r][t] = f32x4{0.f, 0.f, 0.f, 0.f};

    {
        // Software pipeline of depth D.  Every load of the steady-state loop is unconditional (the
        // index is clamped to the range, a clamped load re-reads the last tile) so that the compiler
        // can count the loads in flight and wait only for the oldest slot.
        u32x4 a[D][R], b[D][2 * T];
#pragma unroll
        for (int d = 0; d < D; ++d) {
            const int kt = min(kw0 + d, kw1 - 1);
#pragma unroll
            for (int r = 0; r < R; ++r) a[d][r] = load_weight_tile<T>(wp[r] + (size_t)(kt - kw0) * wstep);
#pragma unroll
            for (int t = 0; t < 2 * T; ++t) b[d][t] = xp[kt * xkt + boff[t]];
        }
        int kt = kw0;
        for (; kt + D <= kw1; kt += D) {
#pragma unroll
            for (int d = 0; d < D; ++d) {
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int t = 0; t < T; ++t) acc[r][t] = mfma16(a[d][r], b[d][2 * t], acc[r][t]);
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int t = 0; t < T; ++t) acc[r][t] = mfma16(a[d][r], b[d][2 * t + 1], acc[r][t]);
                const int nk = min(kt + d + D, kw1 - 1);
#pragma unroll
                for (int r = 0; r < R; ++r) a[d][r] = load_weight_tile<T>(wp[r] + (size_t)(nk - kw0) * wstep);
#pragma unroll
                for (int t = 0; t < 2 * T; ++t) b[d][t] = xp[nk * xkt + boff[t]];
                // keep the refill of slot d right behind its MFMAs: the scheduler would otherwise sink
                // all loads to the end of the body and drain the pipeline once per iteration
                __builtin_amdgcn_sched_barrier(0);
            }
        }
#pragma unroll
        for (int d = 0; d < D; ++d) {  // the last span % D tiles, already in flight
            if (kt + d < kw1) {
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int t = 0; t < T; ++t) {
                        acc[r][t] = mfma16(a[d][r], b[d][2 * t], acc[r][t]);
                        acc[r][t] = mfma16(a[d][r], b[d][2 * t + 1], acc[r][t]);
                    }
            }
        }
    }

    // Cross-wave reduction through LDS in a fixed order (wave 0 + 1 + 2 + 3): all R * T tiles at once
    // while they fit 144 KB, in two halves beyond (8 weight tiles x 5-6 row tiles).
    constexpr int RC = (R * T <= 36) ? R : R / 2;
    static_assert(RC * T <= 36 && R % RC == 0 && RC % 2 == 0, "reduction buffer");
    __shared__ f32x4 red[4][RC * T][64];
    const int N = g.w.n;
    float best = -INFINITY;  // EPI_ARGMAX: running (max, lowest index) of row threadIdx.x
    int bidx = INT_MAX;
#pragma unroll
    for (int rc0 = 0; rc0 < R; rc0 += RC) {
        if (rc0 > 0) __syncthreads();
#pragma unroll
        for (int r = 0; r < RC; ++r)
#pragma unroll
            for (int t = 0; t < T; ++t) red[wave][r * T + t][lane] = acc[rc0 + r][t];
        __syncthreads();

        if (EPI == EPI_F32 || EPI == EPI_ARGMAX) {
            float* outp = g.out ? g.out + (size_t)s * g.split_stride + (size_t)pass * 16 * T * g.ldo : nullptr;
            const bool vec_ok = (g.ldo & 3) == 0;
            for (int i = threadIdx.x; i < RC * T * 64; i += 256) {
                const int rt = i >> 6, l = i & 63;
                const int r = rt / T, t = rt % T;
                const f32x4 v = red[0][rt][l] + red[1][rt][l] + red[2][rt][l] + red[3][rt][l];
                if (EPI == EPI_ARGMAX) red[0][rt][l] = v;
                const int nt = nt0 + rc0 + r;
                const int tok = 16 * t + (l & 15);
                if (nt >= g.w.n_tiles || tok >= m_rows || !outp) continue;
                const int n = nt * 16 + 4 * (l >> 4);
                float* o = outp + (size_t)tok * g.ldo + n;
                if (vec_ok && n + 3 < N) {
                    *(f32x4*)o = v;
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (n + e < N) o[e] = v[e];
                }
            }
            if (EPI == EPI_ARGMAX) {  // per row the (max, lowest index) pair over this workgroup's columns
                __syncthreads();
                const int tok = threadIdx.x;
                if (tok < T * 16 && tok < m_rows) {
                    const int t = tok >> 4, c = tok & 15;
                    for (int r = 0; r < RC; ++r) {
                        const int nt = nt0 + rc0 + r;
                        if (nt >= g.w.n_tiles) break;
                        for (int q = 0; q < 4; ++q) {
                            const f32x4 v = red[0][r * T + t][q * 16 + c];
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                const int n = nt * 16 + 4 * q + e;
                                if (n < N && v[e] > best) { best = v[e]; bidx = n; }
                            }
                        }
                    }
                }
            }
        } else {  // EPI_SWIGLU: even tiles are gate rows, odd tiles the matching up rows
            for (int i = threadIdx.x; i < (RC / 2) * T * 64; i += 256) {
                const int pt = i >> 6, l = i & 63;
                const int p = pt / T, t = pt % T;
                const int tok = 16 * t + (l & 15);
                if (tok >= m_rows) continue;
                const int m = row_tile0 * 16 + tok;
                const int ga = (2 * p) * T + t, ua = (2 * p + 1) * T + t;
                const f32x4 gt = red[0][ga][l] + red[1][ga][l] + red[2][ga][l] + red[3][ga][l];
                const f32x4 up = red[0][ua][l] + red[1][ua][l] + red[2][ua][l] + red[3][ua][l];
                const int j = (((nt0 + rc0) >> 1) + p) * 16 + 4 * (l >> 4);
                uint32_t hi[4], lo[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    // silu(g) * u with the hardware exp2 / reciprocal (about 1 ulp each)
                    const float gg = gt[e];
                    const float v = gg * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * gg)) * up[e];
                    const uint16_t h = f2bf(v);
                    hi[e] = h;
                    lo[e] = f2bf(v - bf2f(h));
                }
                if (j + 3 < g.ffn) {
                    *(u32x2*)(g.h + xt_index(m, j, g.xs, 0)) = u32x2{hi[0] | (hi[1] << 16), hi[2] | (hi[3] << 16)};
                    *(u32x2*)(g.h + xt_index(m, j, g.xs, 1)) = u32x2{lo[0] | (lo[1] << 16), lo[2] | (lo[3] << 16)};
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        if (j + e < g.ffn) {
                            g.h[xt_index(m, j + e, g.xs, 0)] = (uint16_t)hi[e];
                            g.h[xt_index(m, j + e, g.xs, 1)] = (uint16_t)lo[e];
                        }
                    }
                }
            }
        }
    }
    if (EPI == EPI_ARGMAX) {
        const int tok = threadIdx.x;
        if (tok < T * 16 && tok < m_rows) {
            g.arg_val[(size_t)(pass * 16 * T + tok) * g.arg_groups + bx] = best;
            g.arg_idx[(size_t)(pass * 16 * T + tok) * g.arg_groups + bx] = bidx;
        }
    }
}

// Every wave takes all r_pack weight tiles of its group, whatever the number of row tiles.
int gemm_tiles_per_wave(const PackedW& w, int total_rows) {
    (void)total_rows;
    return w.r_pack;
}
int gemm_groups(const PackedW& w, int tiles_per_wave) { return w.groups * w.r_pack / tiles_per_wave; }

template <int EPI, int R, int D>
static hipError_t launch_gemm_small(const GemmLaunch& g, hipStream_t s) {  // at most 3 row tiles
    const dim3 grid(gemm_groups(g.w, R), g.w.splits), block(256);
    switch (ceil_div(g.m, 16)) {
        case 1: hipLaunchKernelGGL((gemm_skinny_kernel<1, R, EPI, D>), grid, block, 0, s, g); break;
        case 2: hipLaunchKernelGGL((gemm_skinny_kernel<2, R, EPI, D>), grid, block, 0, s, g); break;
        case 3: hipLaunchKernelGGL((gemm_skinny_kernel<3, R, EPI, D>), grid, block, 0, s, g); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

template <int EPI, int R>
static hipError_t launch_gemm_large(const GemmLaunch& g, hipStream_t s) {  // 4 to 6 row tiles per pass
    const dim3 block(256);
    dim3 grid(gemm_groups(g.w, R), g.w.splits);
    if (g.passes > 1) grid = dim3(8 * ceil_div(gemm_groups(g.w, R) * g.w.splits, 8) * g.passes);
    switch (g.passes > 1 ? kMaxRowTiles : ceil_div(g.m, 16)) {
        case 4: hipLaunchKernelGGL((gemm_skinny_kernel<4, R, EPI, 2>), grid, block, 0, s, g); break;
        case 5: hipLaunchKernelGGL((gemm_skinny_kernel<5, R, EPI, 2>), grid, block, 0, s, g); break;
        case 6: hipLaunchKernelGGL((gemm_skinny_kernel<6, R, EPI, 2>), grid, block, 0, s, g); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

template <int EPI>
static hipError_t launch_gemm_t(const GemmLaunch& g, hipStream_t s) {
    const int T = g.passes > 1 ? kMaxRowTiles : ceil_div(g.m, 16);
    if (T <= 3) {
        switch (g.tiles_per_wave) {
            case 2: return launch_gemm_small<EPI, 2, 3>(g, s);
            case 4: return launch_gemm_small<EPI, 4, 3>(g, s);
            case 6: return launch_gemm_small<EPI, 6, 3>(g, s);
            case 8: return launch_gemm_small<EPI, 8, 3>(g, s);
            default: return hipErrorInvalidValue;
        }
    }
    switch (g.tiles_per_wave) {
        case 2: return launch_gemm_large<EPI, 2>(g, s);
        case 4: return launch_gemm_large<EPI, 4>(g, s);
        case 6: return launch_gemm_large<EPI, 6>(g, s);
        case 8: return launch_gemm_large<EPI, 8>(g, s);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_gemm(const GemmLaunch& g, GemmEpilogue epi, hipStream_t s) {
    if (g.passes < 1 || g.m < 1 || g.m > 16 * kMaxRowTiles * g.passes || g.w.splits < 1 || g.w.lq < 1)
        return hipErrorInvalidValue;
    if (g.passes > 1 && (g.m <= 16 * kMaxRowTiles * (g.passes - 1) || g.row_tile0 != 0)) return hipErrorInvalidValue;
    if (epi != EPI_F32 && g.w.splits != 1) return hipErrorInvalidValue;
    if (g.row_tile0 < 0 || g.row_tile0 + ceil_div(g.m, 16) > g.xs.row_tiles || g.xs.last_cols < 1 || g.xs.last_cols > 16) return hipErrorInvalidValue;
    if (g.tiles_per_wave > g.w.r_pack || g.w.r_pack % g.tiles_per_wave) return hipErrorInvalidValue;
    switch (epi) {
        case EPI_F32: return launch_gemm_t<EPI_F32>(g, s);
        case EPI_SWIGLU: return launch_gemm_t<EPI_SWIGLU>(g, s);
        case EPI_ARGMAX: return launch_gemm_t<EPI_ARGMAX>(g, s);
    }
    return hipErrorInvalidValue;
}

// ------------------------------------------------------------------------------------------
// rotary table (once, at init), embedding gather + position ids + first RMSNorm (once per step)
// ------------------------------------------------------------------------------------------
// position id of a row = committed length + (#visible in-block keys - 1)  (text after Eq. 3)

// cos / sin of pos * base^(-2i/head_dim) for every position the context can hold, in double
__global__ __launch_bounds__(64) void rope_table_kernel(float* cos_t, float* sin_t, int n_pos, int head_dim, float rope_base) {
    const int pos = blockIdx.x, half = head_dim >> 1;
    for (int i = threadIdx.x; i < half; i += 64) {
        const double inv_freq = pow((double)rope_base, -2.0 * (double)i / (double)head_dim);
        const double ang = (double)pos * inv_freq;
        cos_t[(size_t)pos * half + i] = (float)cos(ang);
        sin_t[(size_t)pos * half + i] = (float)sin(ang);
    }
}

hipError_t launch_rope_table(float* cos_t, float* sin_t, int n_pos, int head_dim, float rope_base, hipStream_t s) {
    if (n_pos < 1) return hipErrorInvalidValue;
    hipLaunchKernelGGL(rope_table_kernel, dim3(n_pos), dim3(64), 0, s, cos_t, sin_t, n_pos, head_dim, rope_base);
    return hipGetLastError();
}

// Row of workgroup i in the one-row-per-workgroup launches below.  Workgroups go to the 8 XCDs in turn and
// every XCD has an L2 of its own; in the operand planes 8 consecutive rows share each 128-byte line (16
// bytes per row).  Rows 8g .. 8g+7 are therefore given to workgroups 8 apart -- the same XCD -- so that one
// L2 collects whole lines instead of eight of them writing back an eighth each.  Grids are rounded up to 64.
__device__ __forceinline__ int xcd_grouped_row(int i) { return (((i >> 6) * 8 + (i & 7)) << 3) + ((i >> 3) & 7); }

// Second half of a normalisation launch: block-wide sum of squares of the row held in v (one float4 per
// thread, two when d_model > 4096), then x * rsqrt(mean + eps) * w as hi / lo operand planes.
// (the norm weights are requested by the caller, with the row itself: asked for here, behind the barrier,
// they cost the kernel a second memory round trip)
__device__ __forceinline__ void norm_w_load(const uint16_t* __restrict__ w, int d, u32x2 (&wv)[2]) {
    const int nvec = d >> 2, nthr = blockDim.x;
#pragma unroll
    for (int c = 0; c < 2; ++c) {
        const int i = threadIdx.x + c * nthr;
        wv[c] = i < nvec ? *(const u32x2*)(w + 4 * i) : u32x2{0, 0};
    }
}
__device__ __forceinline__ void norm_row_tail(const f32x4 (&v)[2], float ss, float* sh, const u32x2 (&wvs)[2],
                                              float eps, int d, int row, uint16_t* __restrict__ xn, XtShape xs) {
    const int nvec = d >> 2, nthr = blockDim.x;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = ss;
    __syncthreads();
    float tot = 0.f;
    for (int i = 0; i < (nthr >> 6); ++i) tot += sh[i];
    const float rs = 1.0f / sqrtf(tot / (float)d + eps);
#pragma unroll
    for (int c = 0; c < 2; ++c) {
        const int i = threadIdx.x + c * nthr;
        if (i < nvec) {
            const u32x2 wv = wvs[c];
            const float wf[4] = {bf2f((uint16_t)(wv[0] & 0xFFFF)), bf2f((uint16_t)(wv[0] >> 16)),
                                 bf2f((uint16_t)(wv[1] & 0xFFFF)), bf2f((uint16_t)(wv[1] >> 16))};
            uint32_t hi[4], lo[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float y = v[c][e] * rs * wf[e];
                const uint16_t h = f2bf(y);
                hi[e] = h;
                lo[e] = f2bf(y - bf2f(h));
            }
            *(u32x2*)(xn + xt_index(row, 4 * i, xs, 0)) = u32x2{hi[0] | (hi[1] << 16), hi[2] | (hi[3] << 16)};
            *(u32x2*)(xn + xt_index(row, 4 * i, xs, 1)) = u32x2{lo[0] | (lo[1] << 16), lo[2] | (lo[3] << 16)};
        }
    }
}

// One workgroup per block row: the embedding row (the mask embedding on mask rows) becomes the residual
// stream, the row's position id and its rotary factors (out of the table) are noted, and the first
// layer's RMSNorm goes with it -- one launch instead of two at the head of every step.
__global__ __launch_bounds__(1024) void embed_kernel(const int32_t* tokens, const uint16_t* embed, int vocab, int d,
                                                     const int32_t* info, const int32_t* rel_pos, int L, int m,
                                                     const int32_t* kv_len, const float* __restrict__ cos_tab,
                                                     const float* __restrict__ sin_tab, int n_pos, int head_dim,
                                                     float* x, int32_t* pos_out, float* cos_t, float* sin_t, int32_t* faults,
                                                     const uint16_t* __restrict__ w, float eps, uint16_t* __restrict__ xn,
                                                     XtShape xs) {
    __shared__ float sh[16];
    const int row = xcd_grouped_row(blockIdx.x), nvec = d >> 2, nthr = blockDim.x;
    if (row >= m) return;  // whole workgroup
    u32x2 wv[2];
    norm_w_load(w, d, wv);
    const int b = row / L, r = row % L;
    int tok = tokens[row];
    if (info[r] & 1) {
        tok = vocab;  // mask rows use the mask embedding whatever the id says
    } else if (tok < 0 || tok > vocab) {
        if (threadIdx.x == 0) atomicAdd(faults, 1);
        tok = min(max(tok, 0), vocab);
    }
    const int pos = kv_len[b] + rel_pos[r];
    if (threadIdx.x == 0) pos_out[row] = pos;
    const int half = head_dim >> 1, tp = min(max(pos, 0), n_pos - 1);
    for (int i = threadIdx.x; i < half; i += nthr) {
        cos_t[(size_t)row * half + i] = cos_tab[(size_t)tp * half + i];
        sin_t[(size_t)row * half + i] = sin_tab[(size_t)tp * half + i];
    }
    const uint16_t* e = embed + (size_t)tok * d;
    f32x4* xr = (f32x4*)(x + (size_t)row * d);
    f32x4 v[2];
    float ss = 0.f;
#pragma unroll
    for (int c = 0; c < 2; ++c) {
        const int i = threadIdx.x + c * nthr;
        v[c] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (i < nvec) {
            const u32x2 ev = *(const u32x2*)(e + 4 * i);
            const f32x4 val = {bf2f((uint16_t)(ev[0] & 0xFFFF)), bf2f((uint16_t)(ev[0] >> 16)),
                               bf2f((uint16_t)(ev[1] & 0xFFFF)), bf2f((uint16_t)(ev[1] >> 16))};
            xr[i] = val;
            v[c] = val;
            ss += val[0] * val[0] + val[1] * val[1] + val[2] * val[2] + val[3] * val[3];
        }
    }
    norm_row_tail(v, ss, sh, wv, eps, d, row, xn, xs);
}

hipError_t launch_embed(const int32_t* tokens, const uint16_t* embed, int vocab, int d, const LayoutDev& lay,
                        const int32_t* kv_len, int batch, const float* cos_tab, const float* sin_tab, int n_pos,
                        int head_dim, float* x, int32_t* pos, float* cos_t, float* sin_t, int32_t* faults,
                        const uint16_t* norm_w, float eps, uint16_t* xn, XtShape xs, hipStream_t s) {
    if (d > 8192 || (d & 3) || n_pos < 1) return hipErrorInvalidValue;
    const int nvec = d >> 2;
    const int threads = nvec >= 1024 ? 1024 : round_up(nvec, 64);
    hipLaunchKernelGGL(embed_kernel, dim3(round_up(batch * lay.L, 64)), dim3(threads), 0, s, tokens, embed, vocab, d, lay.info,
                       lay.rel_pos, lay.L, batch * lay.L, kv_len, cos_tab, sin_tab, n_pos, head_dim, x, pos, cos_t, sin_t, faults,
                       norm_w, eps, xn, xs);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// residual add of split partials + RMSNorm -> hi/lo operand planes of the next projection
// ------------------------------------------------------------------------------------------

// One workgroup per row, one float4 per thread (two when d_model > 4096); all loads of a thread
// are independent so that the kernel costs one memory round trip, not one per split.
__global__ __launch_bounds__(1024) void resid_norm_kernel(float* __restrict__ x, const float* __restrict__ part,
                                                          int splits, size_t split_stride, int ldp,
                                                          const uint16_t* __restrict__ w, float eps, int m, int d,
                                                          uint16_t* __restrict__ xn, XtShape xs) {
    __shared__ float sh[16];
    const int row = xcd_grouped_row(blockIdx.x), nvec = d >> 2, nthr = blockDim.x;
    if (row >= m) return;  // whole workgroup
    u32x2 wv[2];
    norm_w_load(w, d, wv);
    f32x4* xr = (f32x4*)(x + (size_t)row * d);
    f32x4 v[2];
    float ss = 0.f;
#pragma unroll
    for (int c = 0; c < 2; ++c) {
        const int i = threadIdx.x + c * nthr;
        v[c] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (i < nvec) {
            f32x4 val = xr[i];
            f32x4 p[8];
#pragma unroll
            for (int s = 0; s < 8; ++s)
                p[s] = s < splits ? *(const f32x4*)(part + (size_t)s * split_stride + (size_t)row * ldp + 4 * i)
                                  : f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < 8; ++s) val += p[s];
            if (splits > 0) xr[i] = val;
            v[c] = val;
            ss += val[0] * val[0] + val[1] * val[1] + val[2] * val[2] + val[3] * val[3];
        }
    }
    norm_row_tail(v, ss, sh, wv, eps, d, row, xn, xs);
}

hipError_t launch_resid_norm(float* x, const float* part, int splits, size_t split_stride, int ldp,
                             const uint16_t* w, float eps, int m, int d, uint16_t* xn, XtShape xs, hipStream_t s) {
    if (d > 8192 || (d & 3) || (ldp & 3) || splits > 8) return hipErrorInvalidValue;
    const int nvec = d >> 2;
    const int threads = nvec >= 1024 ? 1024 : round_up(nvec, 64);
    hipLaunchKernelGGL(resid_norm_kernel, dim3(round_up(m, 64)), dim3(threads), 0, s, x, part, splits, split_stride, ldp, w, eps,
                       m, d, xn, xs);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// rotary embedding of q, k + store of q (hi/lo planes), block K/V and (non-mask rows) cache K/V in bf16
// ------------------------------------------------------------------------------------------
// Non-mask row of group g sits at position len + g, which is also the cache slot it takes when a
// later commit accepts it, so it is written there right away; mask rows only go to the block
// staging buffers.

__global__ __launch_bounds__(64) void rope_store_kernel(RopeStore a) {
    const int row = blockIdx.x, h = blockIdx.y;
    const int b = row / a.L, r = row % a.L;
    const int H = a.n_heads, Hkv = a.n_kv_heads, dh = a.head_dim, half = dh >> 1;
    const int hd = H * dh, ld = (H + 2 * Hkv) * dh;
    const bool is_mask = a.info[r] & 1;
    const int slot = a.pos[row];
    const bool to_cache = !is_mask && slot >= 0 && slot < a.capacity;
    if (!is_mask && !to_cache && threadIdx.x == 0 && h == 0) atomicAdd(a.faults, 1);
    const int Lb = a.Lp / kAttnKeys;
    const int i = threadIdx.x;
    if (i >= half) return;
    const bool kv_head = h < Hkv;  // block (row, h) also handles key/value head h
    float q0 = 0.f, q1 = 0.f, k0 = 0.f, k1 = 0.f, v0 = 0.f, v1 = 0.f;
    const float* __restrict__ base = a.qkv + (size_t)row * ld + h * dh + i;
#pragma unroll
    for (int s = 0; s < 8; ++s) {
        if (s < a.splits) {
            const float* p = base + (size_t)s * a.split_stride;
            q0 += p[0]; q1 += p[half];
            if (kv_head) {
                k0 += p[hd]; k1 += p[hd + half];
                v0 += p[hd + Hkv * dh]; v1 += p[hd + Hkv * dh + half];
            }
        }
    }
    const float c = a.cos_t[(size_t)row * half + i], sn = a.sin_t[(size_t)row * half + i];
    const float qra = q0 * c - q1 * sn, qrb = q1 * c + q0 * sn;
    const uint16_t qa = f2bf(qra), qb = f2bf(qrb);
    uint16_t* qo = a.q + (((size_t)b * H + h) * a.L + r) * dh;
    qo[i] = qa; qo[i + half] = qb;
    qo[a.q_plane + i] = f2bf(qra - bf2f(qa)); qo[a.q_plane + i + half] = f2bf(qrb - bf2f(qb));
    if (!kv_head) return;
    const uint16_t ka = f2bf(k0 * c - k1 * sn), kb = f2bf(k1 * c + k0 * sn);
    const uint16_t va = f2bf(v0), vb = f2bf(v1);
    const size_t bh = (size_t)b * Hkv + h;
    uint16_t* ko = a.kblk + (bh * a.Lp + r) * dh;
    ko[i] = ka; ko[i + half] = kb;
    uint16_t* vo = a.vblk + ((bh * Lb + r / kAttnKeys) * dh) * kAttnKeys + (r % kAttnKeys);
    vo[(size_t)i * kAttnKeys] = va; vo[(size_t)(i + half) * kAttnKeys] = vb;
    if (to_cache) {
        bool bad = false;
        const size_t run = a.paging.table
                               ? kv_run_offset<true>(a.paging, b, h, Hkv, a.capacity, dh, slot / kAttnKeys, &bad)
                               : kv_run_offset<false>(a.paging, b, h, Hkv, a.capacity, dh, slot / kAttnKeys);
        if (bad && i == 0) atomicAdd(a.faults, 1);
        uint16_t* kc = a.kc + run + (size_t)(slot % kAttnKeys) * dh;
        kc[i] = ka; kc[i + half] = kb;
        uint16_t* vc = a.vc + run + (slot % kAttnKeys);
        vc[(size_t)i * kAttnKeys] = va; vc[(size_t)(i + half) * kAttnKeys] = vb;
    }
}

// The same for long blocks (prompt chunks, batches of large blocks): one workgroup per (32 rows of a
// sequence, head).  A thread takes items of 4 rotary pairs (columns i..i+3 and i+half..i+half+3 of one
// row; two items at head size 128) and requests everything they need -- every partial sum, the rotary
// factors, the row's slot -- before it uses any of it: taking the rows in turn, a load and its use per
// row, spent a memory round trip on each (33 us for 1024 rows of a 7B layer).  V goes to an LDS tile first
// and leaves it transposed, 32 rows of one dimension side by side: written straight from the items every
// 2-byte element of V would open a 64-byte line of its own.
template <int DH>
__global__ __launch_bounds__(256) void rope_store_rows_kernel(RopeStore a) {
    constexpr int half = DH / 2, IPR = half / 4, NI = kAttnKeys * IPR / 256;
    static_assert(kAttnKeys * IPR % 256 == 0, "whole items per thread");
    typedef __attribute__((ext_vector_type(4))) float f4;
    const int tid = threadIdx.x;
    const int h = blockIdx.y;
    const int n_chunk = a.Lp / kAttnKeys;
    const int b = blockIdx.x / n_chunk, ch = blockIdx.x % n_chunk;
    const int r0 = ch * kAttnKeys;
    const int H = a.n_heads, Hkv = a.n_kv_heads;
    const int hd = H * DH, ld = (H + 2 * Hkv) * DH;
    const bool kv_head = h < Hkv;  // whole workgroup
    __shared__ uint16_t v_tile[DH][kAttnKeys + 2];
    __shared__ int s_slot[kAttnKeys];  // cache slot of the row, -1: not cached
    const size_t bh = (size_t)b * Hkv + h;
    const size_t ss = a.split_stride;

    int it_rr[NI], it_i[NI], it_slot[NI];
    bool it_on[NI], it_mask[NI];
    const float* qp[NI];
    f4 cs[NI], sn[NI], q0[NI], q1[NI], k0[NI], k1[NI], v0[NI], v1[NI];
#pragma unroll
    for (int it = 0; it < NI; ++it) {
        const int u = tid + it * 256;
        it_rr[it] = u / IPR;
        it_i[it] = (u % IPR) * 4;
        it_on[it] = r0 + it_rr[it] < a.L;
        const int rc = min(r0 + it_rr[it], a.L - 1), row = b * a.L + rc;  // rows past the block: a real row, dropped below
        qp[it] = a.qkv + (size_t)row * ld + h * DH + it_i[it];
        cs[it] = *(const f4*)(a.cos_t + (size_t)row * half + it_i[it]);
        sn[it] = *(const f4*)(a.sin_t + (size_t)row * half + it_i[it]);
        it_mask[it] = a.info[rc] & 1;
        it_slot[it] = a.pos[row];
    }
    const f4 z4 = {0.f, 0.f, 0.f, 0.f};
    // S partial sums at once, the rest (if any) in rounds of one
    auto sums = [&](auto S_) {
        constexpr int S = decltype(S_)::value;
        f4 tq0[NI][S], tq1[NI][S], tk0[NI][S], tk1[NI][S], tv0[NI][S], tv1[NI][S];
#pragma unroll
        for (int it = 0; it < NI; ++it)
#pragma unroll
            for (int sp = 0; sp < S; ++sp) {
                tq0[it][sp] = *(const f4*)(qp[it] + sp * ss);
                tq1[it][sp] = *(const f4*)(qp[it] + sp * ss + half);
            }
        if (kv_head) {
#pragma unroll
            for (int it = 0; it < NI; ++it)
#pragma unroll
                for (int sp = 0; sp < S; ++sp) {
                    tk0[it][sp] = *(const f4*)(qp[it] + sp * ss + hd);
                    tk1[it][sp] = *(const f4*)(qp[it] + sp * ss + hd + half);
                    tv0[it][sp] = *(const f4*)(qp[it] + sp * ss + hd + Hkv * DH);
                    tv1[it][sp] = *(const f4*)(qp[it] + sp * ss + hd + Hkv * DH + half);
                }
        }
#pragma unroll
        for (int it = 0; it < NI; ++it) {
            q0[it] = q1[it] = k0[it] = k1[it] = v0[it] = v1[it] = z4;
#pragma unroll
            for (int sp = 0; sp < S; ++sp) { q0[it] += tq0[it][sp]; q1[it] += tq1[it][sp]; }
        }
        if (kv_head) {
#pragma unroll
            for (int it = 0; it < NI; ++it)
#pragma unroll
                for (int sp = 0; sp < S; ++sp) {
                    k0[it] += tk0[it][sp]; k1[it] += tk1[it][sp];
                    v0[it] += tv0[it][sp]; v1[it] += tv1[it][sp];
                }
        }
        for (int sp = S; sp < a.splits; ++sp) {
            f4 t0[NI], t1[NI], t2[NI], t3[NI], t4[NI], t5[NI];
#pragma unroll
            for (int it = 0; it < NI; ++it) {
                t0[it] = *(const f4*)(qp[it] + sp * ss);
                t1[it] = *(const f4*)(qp[it] + sp * ss + half);
            }
            if (kv_head) {
#pragma unroll
                for (int it = 0; it < NI; ++it) {
                    t2[it] = *(const f4*)(qp[it] + sp * ss + hd);
                    t3[it] = *(const f4*)(qp[it] + sp * ss + hd + half);
                    t4[it] = *(const f4*)(qp[it] + sp * ss + hd + Hkv * DH);
                    t5[it] = *(const f4*)(qp[it] + sp * ss + hd + Hkv * DH + half);
                }
            }
#pragma unroll
            for (int it = 0; it < NI; ++it) { q0[it] += t0[it]; q1[it] += t1[it]; }
            if (kv_head) {
#pragma unroll
                for (int it = 0; it < NI; ++it) { k0[it] += t2[it]; k1[it] += t3[it]; v0[it] += t4[it]; v1[it] += t5[it]; }
            }
        }
    };
    if (a.splits == 2) sums(std::integral_constant<int, 2>{});
    else sums(std::integral_constant<int, 1>{});

#pragma unroll
    for (int it = 0; it < NI; ++it) {
        const int rr = it_rr[it], i = it_i[it], r = r0 + rr;
        const int slot = it_slot[it];
        const bool to_cache = it_on[it] && !it_mask[it] && slot >= 0 && slot < a.capacity;
        if (i == 0) {
            s_slot[rr] = to_cache ? slot : -1;
            if (it_on[it] && !it_mask[it] && !to_cache && h == 0) atomicAdd(a.faults, 1);
        }
        if (!it_on[it]) continue;
        uint32_t ah[4], al[4], bh_[4], bl[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float ra = q0[it][e] * cs[it][e] - q1[it][e] * sn[it][e], rb = q1[it][e] * cs[it][e] + q0[it][e] * sn[it][e];
            const uint16_t ha = f2bf(ra), hb = f2bf(rb);
            ah[e] = ha; al[e] = f2bf(ra - bf2f(ha));
            bh_[e] = hb; bl[e] = f2bf(rb - bf2f(hb));
        }
        uint16_t* qo = a.q + (((size_t)b * H + h) * a.L + r) * DH + i;
        *(u32x2*)qo = u32x2{ah[0] | (ah[1] << 16), ah[2] | (ah[3] << 16)};
        *(u32x2*)(qo + half) = u32x2{bh_[0] | (bh_[1] << 16), bh_[2] | (bh_[3] << 16)};
        *(u32x2*)(qo + a.q_plane) = u32x2{al[0] | (al[1] << 16), al[2] | (al[3] << 16)};
        *(u32x2*)(qo + a.q_plane + half) = u32x2{bl[0] | (bl[1] << 16), bl[2] | (bl[3] << 16)};
        if (!kv_head) continue;
        uint32_t ka[4], kb[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            ka[e] = f2bf(k0[it][e] * cs[it][e] - k1[it][e] * sn[it][e]);
            kb[e] = f2bf(k1[it][e] * cs[it][e] + k0[it][e] * sn[it][e]);
            v_tile[i + e][rr] = f2bf(v0[it][e]);
            v_tile[i + e + half][rr] = f2bf(v1[it][e]);
        }
        const u32x2 kav = {ka[0] | (ka[1] << 16), ka[2] | (ka[3] << 16)};
        const u32x2 kbv = {kb[0] | (kb[1] << 16), kb[2] | (kb[3] << 16)};
        uint16_t* ko = a.kblk + (bh * a.Lp + r) * DH + i;
        *(u32x2*)ko = kav;
        *(u32x2*)(ko + half) = kbv;
        if (to_cache) {
            bool bad = false;
            const size_t run = a.paging.table
                                   ? kv_run_offset<true>(a.paging, b, h, Hkv, a.capacity, DH, slot / kAttnKeys, &bad)
                                   : kv_run_offset<false>(a.paging, b, h, Hkv, a.capacity, DH, slot / kAttnKeys);
            if (bad && i == 0) atomicAdd(a.faults, 1);
            uint16_t* kc = a.kc + run + (size_t)(slot % kAttnKeys) * DH + i;
            *(u32x2*)kc = kav;
            *(u32x2*)(kc + half) = kbv;
        }
    }
    if (!kv_head) return;  // whole workgroup
    __syncthreads();
    // V: thread t takes row t % 32 of dimensions t / 32, t / 32 + 8, ...: a wave writes two runs of 32 rows
    const int rr = tid & 31, r = r0 + rr;
    const int slot = s_slot[rr];
    size_t run = 0;
    if (slot >= 0)
        run = a.paging.table ? kv_run_offset<true>(a.paging, b, h, Hkv, a.capacity, DH, slot / kAttnKeys)
                             : kv_run_offset<false>(a.paging, b, h, Hkv, a.capacity, DH, slot / kAttnKeys);
    uint16_t* vo = a.vblk + ((bh * n_chunk + ch) * DH) * kAttnKeys + rr;
    uint16_t* vc = a.vc + run + (slot % kAttnKeys);
    for (int d = tid >> 5; d < DH; d += 8) {
        if (r >= a.L) continue;
        const uint16_t v = v_tile[d][rr];
        vo[(size_t)d * kAttnKeys] = v;
        if (slot >= 0) vc[(size_t)d * kAttnKeys] = v;
    }
}

hipError_t launch_rope_store(const RopeStore& a, hipStream_t s) {
    if (a.splits > 8 || a.head_dim > 128 || a.n_kv_heads < 1 || a.n_heads % a.n_kv_heads) return hipErrorInvalidValue;
    if (a.paging.table && (a.paging.table_stride * kAttnKeys != a.capacity || a.paging.n_pages < 1)) return hipErrorInvalidValue;
    if (a.Lp % kAttnKeys || a.Lp < a.L) return hipErrorInvalidValue;
    if (a.L >= 2 * kAttnKeys && a.head_dim == 128)
        hipLaunchKernelGGL(rope_store_rows_kernel<128>, dim3(a.batch * (a.Lp / kAttnKeys), a.n_heads), dim3(256), 0, s, a);
    else if (a.L >= 2 * kAttnKeys && a.head_dim == 64)
        hipLaunchKernelGGL(rope_store_rows_kernel<64>, dim3(a.batch * (a.Lp / kAttnKeys), a.n_heads), dim3(256), 0, s, a);
    else
        hipLaunchKernelGGL(rope_store_kernel, dim3(a.m, a.n_heads), dim3(64), 0, s, a);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// attention under the semi-autoregressive mask (Eq. 3), split over the key axis
// ------------------------------------------------------------------------------------------
// Every cached key is a committed non-mask token that precedes the block, so clause 1 of Eq. 3
// makes it visible to every block row: cache chunks run unmasked.  The block's own keys follow as
// extra chunks with the in-block rule: key j is visible to row i iff j <= i and (j is not a mask,
// or i is a mask of the same group).
//
// Keys are cut into chunks of 32.  A workgroup of 4 waves works on one (sequence, head, group of TQ
// query tiles); wave w of workgroup gx takes chunks gx*4 + w, + 4*n_wg, ... with a running softmax.
// One wave per SIMD leaves 512 registers per lane: the K/V tiles of the current chunk and of the
// next one (loads of chunk j+1 are in flight while chunk j is computed) and the output
// accumulators stay in registers; Q (hi + lo planes) is staged once per workgroup in LDS.  Per chunk:
//   S^T[key, row] = K * Q^T   (A = K rows in the order key(r) = 8*(r/4) + 4*tile + r%4, so that a
//                              lane ends up with 8 consecutive keys of one query row; Q as hi + lo)
//   softmax over keys (log2 domain), running max shared by the 4 lane groups of a row
//   O^T[d, row] += V^T * P^T  (A = 16x32 tile of the transposed-in-runs-of-32 V cache, B = P split
//                              into bf16 hi + lo so that P keeps ~16 mantissa bits)
// The 4 waves then merge their (max, sum, O) through LDS in a fixed order and write one partial
// per workgroup; a second kernel merges the partials of a row and emits the operand planes of
// the output projection.


// 16 bytes at (base + lane_off + const_off): base the same in all lanes (a buffer descriptor in scalar
// registers, unbounded), lane_off per lane, const_off a constant of the instruction or a scalar.
__device__ __forceinline__ u32x4 chunk_load(const uint16_t* base, int lane_off, int const_off) {
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, -1, 0x00020000);
    return __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rs, lane_off, const_off, 0));
}

// WV waves per workgroup: 4, two workgroups to a CU (256 registers each, under half the LDS).  The kernel
// is written for any count; 8 (one workgroup per CU) was measured and is not built: it was ahead only
// while the 4-wave loop spilled registers, and is level with it since (one sequence of 4096 positions
// beside seven short ones 65 against 67.6 us per layer, everything else equal or behind).
template <int DH, int TQ, bool PAGED, bool FUSE, int WV>
__global__ __launch_bounds__(WV * 64, WV == 4 ? 2 : 1) void attn_sar_kernel(AttnLaunch a, float scale_log2e) {
    constexpr int DS = DH / 32, DT = DH / 16;
    constexpr int kPass = DT < 4 ? DT : 4;  // output slices merged per LDS pass, one per wave (the first kPass)
    constexpr bool kLoopCacheOnly = FUSE;   // the pipelined loop never meets one of the block's own chunks
    const int lane = threadIdx.x & 63, c16 = lane & 15, g4 = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int h = blockIdx.y;
    const int L = a.L, H = a.n_heads;
    const int QG = (((L + 15) >> 4) + TQ - 1) / TQ;
    // query groups in descending order: the later a group sits in a long block the more in-block chunks
    // it has, and the workgroups that take longest should start first
    const int b = blockIdx.z / QG, qg = QG - 1 - blockIdx.z % QG;
    const int r0 = qg * TQ * 16;
    const size_t bh = (size_t)b * H + h;
    const int n_wg = gridDim.x, wg = blockIdx.x;

    constexpr int kQUnits = 2 * TQ * DS * 64, kRedUnits = WV * kPass * TQ * 64;
    // FUSE: the block's own keys and values stay in LDS (as in attn_head_kernel: padded rows)
    constexpr int kStageRows = FUSE ? (kHeadAttnMaxRows + kAttnKeys - 1) / kAttnKeys * kAttnKeys : kAttnKeys;
    constexpr int KROW = DH + 8, VROW = kAttnKeys + 8;
    // One pool: the Q operand planes, the block's keys and values -- all dead once every wave is through
    // its chunks -- and, from the barrier in front of the merge on, the merge buffer on top of them.  With
    // it the 4-wave kernel stays under half the LDS of a CU, which (with at most 256 registers) lets two
    // workgroups share a CU and keeps the compiler from spreading operands over the accumulation registers
    // (with 8 waves the merge buffer would take 98 KB: one workgroup per CU).
    constexpr int kQBytes = kQUnits * 16, kKBytes = FUSE ? kStageRows * KROW * 2 : 0;
    constexpr int kVBytes = FUSE ? kStageRows / kAttnKeys * DH * VROW * 2 : 0, kRedBytes = kRedUnits * 16;
    constexpr int kPoolBytes = kQBytes + kKBytes + kVBytes > kRedBytes ? kQBytes + kKBytes + kVBytes : kRedBytes;
    static_assert(kQBytes % 16 == 0 && kKBytes % 16 == 0, "LDS pool alignment");
    __shared__ __attribute__((aligned(16))) unsigned char pool[kPoolBytes];
    u32x4* const smem = (u32x4*)pool;                              // Q operand planes [plane][t][ds][lane]
    uint16_t* const k_lds = (uint16_t*)(pool + kQBytes);           // FUSE only
    uint16_t* const v_lds = (uint16_t*)(pool + kQBytes + kKBytes);  // FUSE only
    f32x4* const red = (f32x4*)pool;                               // merge buffer [wave][slice in pass][t][lane]
    __shared__ float m_sh[WV][TQ * 16], l_sh[WV][TQ * 16];
    __shared__ int s_info[FUSE ? 16 * kMaxRowTiles : kMaxBlockRows];

    const int len = min(max(a.kv_len[b], 0), a.capacity);
    // in-block keys past this group's last query row are invisible to all of its rows (Eq. 3 is causal):
    // long blocks (prompt chunks) skip those chunks altogether
    const int n_cache = (len + kAttnKeys - 1) / kAttnKeys, n_blk = (min(L, r0 + TQ * 16) + kAttnKeys - 1) / kAttnKeys;
    // FUSE: the pipelined loop runs over the cache chunks only; the last workgroup along the keys (which
    // the bound the grid was sized for usually leaves without cache chunks) takes the block's own
    const int n_chunks = FUSE ? n_cache : n_cache + n_blk;
    const bool blk_wg = FUSE && wg == n_wg - 1;
    if (wg * WV >= n_chunks && !blk_wg) {
        // the grid is sized for an upper bound of the length: a workgroup past the real end only
        // marks its partial as empty (the merge pass skips it)
        const int tok = r0 + (int)threadIdx.x;
        if (threadIdx.x < TQ * 16 && tok < L) {
            const size_t base = (bh * n_wg + wg) * L + tok;
            a.ml_part[base * 2] = -INFINITY;
            a.ml_part[base * 2 + 1] = 0.f;
        }
        return;
    }
    const int chunk_step = n_wg * WV;
    int chunk = wg * WV + wave;
    // grouped-query attention: query head h reads key/value head h / (H / Hkv)
    const int kvh = h / (H / a.n_kv_heads);
    const size_t bkv = (size_t)b * a.n_kv_heads + kvh;
    const uint16_t* kc_base = a.kc;  // + cache_off(chunk): contiguous run or page of this (sequence, head)
    const uint16_t* vc_base = a.vc;
    auto cache_off = [&](int ch) -> size_t { return kv_run_offset<PAGED>(a.paging, b, kvh, a.n_kv_heads, a.capacity, DH, ch); };
    const uint16_t* kb_base = a.kblk + bkv * a.Lp * DH;
    const uint16_t* vb_base = a.vblk + bkv * a.Lp * DH;

    // Two operand buffers.  Every load is unconditional (a chunk index past the end is clamped to
    // the last chunk and its result ignored) so that the compiler can count the loads in flight.
    u32x4 ak0[2][DS], av0[DT], ak1[2][DS];  // (one value buffer: see the loop)
    int c_0 = 0, kend_0 = 1, c_1 = 0, kend_1 = 1;
    bool blk_0 = false, blk_1 = false;
    // Per-lane element offsets inside a chunk.  K: row 8*(c16/4) + 4*tk + c16%4, columns 8*g4.. of
    // contraction step ds (+ 32*ds); V: row 16*dt + c16 of the transposed run, keys 8*g4...  Chunks
    // are read whole: slots past the end hold stale but finite values (the cache is cleared when it
    // is created) and their scores are discarded below.
#define SPACE_ATTN_LANE_OFFSETS                                                                             \
    /* Byte offsets of the lane inside a chunk.  The chunks are read with buffer loads: the chunk's    */     \
    /* address (the same in all lanes) makes a descriptor in scalar registers and the lane adds one   */     \
    /* 32-bit offset.  With plain pointers the compiler folds the lane offset into a 64-bit address   */     \
    /* per lane, keeps it across the loop and, in the variant with three row tiles, spills it: the    */     \
    /* reload at the head of every round then waits for every load in flight (values of the chunk     */     \
    /* just requested included), which is exactly the latency the loop is built to hide.              */     \
    const int koff = 2 * ((8 * (c16 >> 2) + (c16 & 3)) * DH + 8 * g4);                                      \
    const int voff = 2 * (c16 * kAttnKeys + 8 * g4);
// Where chunk CHUNK lives and what bounds it: KB / VB point at its keys / values, C is its first
// position, KEND the end of what is valid there, BLK says that it is one of the block's own chunks.
#define SPACE_ATTN_PREP(KB, VB, C, KEND, BLK, CHUNK)                                                        \
    do {                                                                                                    \
        const int ch_ = min((CHUNK), n_chunks - 1);                                                         \
        BLK = !kLoopCacheOnly && ch_ >= n_cache; /* known at compile time where the block's chunks come out of LDS */ \
        C = (BLK ? ch_ - n_cache : ch_) * kAttnKeys;                                                        \
        KEND = BLK ? L : len;                                                                               \
        const size_t off_ = BLK ? (size_t)C * DH : cache_off(ch_);                                          \
        KB = (BLK ? kb_base : kc_base) + off_;                                                              \
        VB = (BLK ? vb_base : vc_base) + off_;                                                              \
    } while (0)
#define SPACE_ATTN_LOAD_K(AK, KB)                                                                           \
    do {                                                                                                    \
        _Pragma("unroll") for (int tk = 0; tk < 2; ++tk)                                                    \
            _Pragma("unroll") for (int ds = 0; ds < DS; ++ds)                                               \
                AK[tk][ds] = chunk_load(KB, koff, 8 * tk * DH + 64 * ds);                                   \
    } while (0)
#define SPACE_ATTN_LOAD_V(AV, VB)                                                                           \
    do {                                                                                                    \
        _Pragma("unroll") for (int dt = 0; dt < DT; ++dt)                                                   \
            AV[dt] = chunk_load(VB, voff, dt * 32 * kAttnKeys);                                             \
    } while (0)
#define SPACE_ATTN_LOAD(AK, AV, C, KEND, BLK, CHUNK)                                                        \
    do {                                                                                                    \
        const uint16_t *kb_, *vb_;                                                                          \
        SPACE_ATTN_PREP(kb_, vb_, C, KEND, BLK, CHUNK);                                                     \
        SPACE_ATTN_LOAD_K(AK, kb_);                                                                         \
        SPACE_ATTN_LOAD_V(AV, vb_);                                                                         \
    } while (0)

    SPACE_ATTN_LANE_OFFSETS
    // the first chunk is requested before the staging work; FUSE: its values only once the staging work has
    // summed what it requested (registers: everything at once does not fit beside the loop's own)
    const uint16_t *kb0_ = kc_base, *vb0_ = vc_base;
    const bool pre0 = !FUSE || chunk < n_chunks;
    if (pre0) {
        SPACE_ATTN_PREP(kb0_, vb0_, c_0, kend_0, blk_0, chunk);
        SPACE_ATTN_LOAD_K(ak0, kb0_);
        if (!FUSE) SPACE_ATTN_LOAD_V(av0, vb0_);
    }

    int own_info = 0;
    if (!FUSE) {
        // Q planes -> LDS (operand order: lane l = row l%16 of the tile, columns 32*ds + 8*(l/16)..)
        for (int u = threadIdx.x; u < kQUnits; u += WV * 64) {
            const int l = u & 63, ds = (u >> 6) % DS, t = (u / (64 * DS)) % TQ, plane = u / (64 * DS * TQ);
            const int row = min(r0 + 16 * t + (l & 15), L - 1);
            smem[u] = *(const u32x4*)(a.q + (size_t)plane * a.q_plane + (bh * L + row) * DH + 32 * ds + 8 * (l >> 4));
        }
    } else {
        // Work items of 4 rotary pairs (columns i..i+3 and i+half..i+half+3 of one row), as in
        // attn_head_kernel: item u of a thread is row u / (DH/8), columns 4 * (u % (DH/8)); every workgroup
        // rotates the TQ * 16 query rows (rows past the block are zero), the one that takes the block's
        // chunks also the keys and values of the same rows.  Every load is requested before any is
        // consumed (rows past the end are clamped to a real row and their values dropped): this prologue
        // starts while other workgroups stream keys, when a memory round trip takes several microseconds,
        // and with a load per loop pass it paid one for each of them.
        constexpr int half = DH / 2, IPR = half / 4, NTH = WV * 64;
        constexpr int NQI = TQ * 16 * IPR, NI = (NQI + NTH - 1) / NTH;
        typedef __attribute__((ext_vector_type(4))) float f4;
        const int Hkv = a.n_kv_heads, hd = H * DH, ld = (H + 2 * Hkv) * DH;
        const size_t ss = a.split_stride;
        uint16_t* q_lds = (uint16_t*)smem;
        const int tid = threadIdx.x;
        own_info = a.info[min(tid, L - 1)];  // at most 48 rows: one per thread, for the LDS copy below
        const float* qp[NI];
        f4 cs[NI], sn[NI], qs0[NI], qs1[NI], ks0[NI], ks1[NI], vs0[NI], vs1[NI];
        int it_rr[NI], it_i[NI], kv_info[NI], kv_slot[NI];
        bool it_on[NI];
#pragma unroll
        for (int it = 0; it < NI; ++it) {
            const int u = tid + it * NTH, uc = min(u, NQI - 1);
            it_on[it] = u < NQI;
            it_rr[it] = uc / IPR;
            it_i[it] = (uc % IPR) * 4;
            const int row = b * L + min(it_rr[it], L - 1);
            qp[it] = a.qkv + (size_t)row * ld + h * DH + it_i[it];
            cs[it] = *(const f4*)(a.cos_t + (size_t)row * half + it_i[it]);
            sn[it] = *(const f4*)(a.sin_t + (size_t)row * half + it_i[it]);
            kv_info[it] = a.info[min(it_rr[it], L - 1)];
            kv_slot[it] = a.pos[row];
        }
        const int k_off = hd + (kvh - h) * DH, v_off = k_off + Hkv * DH;  // from a row's query columns to its key / value columns
        const f4 z4 = {0.f, 0.f, 0.f, 0.f};
        // SQ / SK partial sums of the queries / of the keys and values are requested at once, the rest
        // (if any) in rounds of one partial sum each
        auto sums = [&](auto SQ_, auto SK_) {
            constexpr int SQ = decltype(SQ_)::value, SK = decltype(SK_)::value;
            f4 tq0[NI][SQ], tq1[NI][SQ], tk0[NI][SK], tk1[NI][SK], tv0[NI][SK], tv1[NI][SK];
#pragma unroll
            for (int it = 0; it < NI; ++it)
#pragma unroll
                for (int sp = 0; sp < SQ; ++sp) {
                    tq0[it][sp] = *(const f4*)(qp[it] + sp * ss);
                    tq1[it][sp] = *(const f4*)(qp[it] + sp * ss + half);
                }
            if (blk_wg) {
#pragma unroll
                for (int it = 0; it < NI; ++it)
#pragma unroll
                    for (int sp = 0; sp < SK; ++sp) {
                        tk0[it][sp] = *(const f4*)(qp[it] + sp * ss + k_off);
                        tk1[it][sp] = *(const f4*)(qp[it] + sp * ss + k_off + half);
                        tv0[it][sp] = *(const f4*)(qp[it] + sp * ss + v_off);
                        tv1[it][sp] = *(const f4*)(qp[it] + sp * ss + v_off + half);
                    }
            }
#pragma unroll
            for (int it = 0; it < NI; ++it) {
                qs0[it] = qs1[it] = z4;
#pragma unroll
                for (int sp = 0; sp < SQ; ++sp) { qs0[it] += tq0[it][sp]; qs1[it] += tq1[it][sp]; }
            }
            if (blk_wg) {
#pragma unroll
                for (int it = 0; it < NI; ++it) {
                    ks0[it] = ks1[it] = vs0[it] = vs1[it] = z4;
#pragma unroll
                    for (int sp = 0; sp < SK; ++sp) {
                        ks0[it] += tk0[it][sp]; ks1[it] += tk1[it][sp];
                        vs0[it] += tv0[it][sp]; vs1[it] += tv1[it][sp];
                    }
                }
            }
            for (int sp = SK; sp < a.splits; ++sp) {
                if (sp >= SQ) {
                    f4 t0[NI], t1[NI];
#pragma unroll
                    for (int it = 0; it < NI; ++it) {
                        t0[it] = *(const f4*)(qp[it] + sp * ss);
                        t1[it] = *(const f4*)(qp[it] + sp * ss + half);
                    }
#pragma unroll
                    for (int it = 0; it < NI; ++it) { qs0[it] += t0[it]; qs1[it] += t1[it]; }
                }
                if (blk_wg) {
                    f4 t2[NI], t3[NI], t4[NI], t5[NI];
#pragma unroll
                    for (int it = 0; it < NI; ++it) {
                        t2[it] = *(const f4*)(qp[it] + sp * ss + k_off);
                        t3[it] = *(const f4*)(qp[it] + sp * ss + k_off + half);
                        t4[it] = *(const f4*)(qp[it] + sp * ss + v_off);
                        t5[it] = *(const f4*)(qp[it] + sp * ss + v_off + half);
                    }
#pragma unroll
                    for (int it = 0; it < NI; ++it) { ks0[it] += t2[it]; ks1[it] += t3[it]; vs0[it] += t4[it]; vs1[it] += t5[it]; }
                }
            }
        };
        typedef std::integral_constant<int, 1> one_t;
        typedef std::integral_constant<int, 2> two_t;
        if (a.splits == 2) {
            sums(two_t{}, std::integral_constant<int, NI < 3 ? 2 : 1>{});
        } else {
            sums(one_t{}, one_t{});
        }
#pragma unroll
        for (int it = 0; it < NI; ++it) {
            if (!it_on[it]) continue;
            const int rr = it_rr[it], i = it_i[it];
            f4 s0 = qs0[it], s1 = qs1[it];
            if (rr >= L) s0 = s1 = z4;
            uint32_t ah[4], al[4], bh_[4], bl[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float ra = s0[e] * cs[it][e] - s1[e] * sn[it][e], rb = s1[e] * cs[it][e] + s0[e] * sn[it][e];
                const uint16_t ha = f2bf(ra), hb = f2bf(rb);
                ah[e] = ha; al[e] = f2bf(ra - bf2f(ha));
                bh_[e] = hb; bl[e] = f2bf(rb - bf2f(hb));
            }
            // element (plane, rr, col) of the planes: ((((plane*TQ + rr/16)*DS + col/32)*64 + rr%16 + 16*((col%32)/8))*8 + col%8
            const int t = rr >> 4, r16 = rr & 15;
            const int qa_i = ((((t * DS + (i >> 5)) * 64) + r16 + 16 * ((i & 31) >> 3)) << 3) + (i & 7);
            const int qb_i = qa_i + (half >> 5) * 64 * 8;
            constexpr int lo_off = TQ * DS * 64 * 8;
            *(u32x2*)(q_lds + qa_i) = u32x2{ah[0] | (ah[1] << 16), ah[2] | (ah[3] << 16)};
            *(u32x2*)(q_lds + qb_i) = u32x2{bh_[0] | (bh_[1] << 16), bh_[2] | (bh_[3] << 16)};
            *(u32x2*)(q_lds + qa_i + lo_off) = u32x2{al[0] | (al[1] << 16), al[2] | (al[3] << 16)};
            *(u32x2*)(q_lds + qb_i + lo_off) = u32x2{bl[0] | (bl[1] << 16), bl[2] | (bl[3] << 16)};
        }
        if (blk_wg) {
            const int group = H / Hkv;
#pragma unroll
            for (int it = 0; it < NI; ++it) {
                const int r = it_rr[it], i = it_i[it];
                if (!it_on[it] || r >= L) continue;
                uint32_t ka[4], kbv_[4];
                uint16_t va[4], vb[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    ka[e] = f2bf(ks0[it][e] * cs[it][e] - ks1[it][e] * sn[it][e]);
                    kbv_[e] = f2bf(ks1[it][e] * cs[it][e] + ks0[it][e] * sn[it][e]);
                    va[e] = f2bf(vs0[it][e]);
                    vb[e] = f2bf(vs1[it][e]);
                }
                const u32x2 kav = {ka[0] | (ka[1] << 16), ka[2] | (ka[3] << 16)};
                const u32x2 kbv = {kbv_[0] | (kbv_[1] << 16), kbv_[2] | (kbv_[3] << 16)};
                uint16_t* ko = k_lds + r * KROW + i;
                *(u32x2*)ko = kav;
                *(u32x2*)(ko + half) = kbv;
                uint16_t* vo = v_lds + ((r / kAttnKeys) * DH + i) * VROW + (r % kAttnKeys);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    vo[e * VROW] = va[e];
                    vo[(e + half) * VROW] = vb[e];
                }
                if (h % group == 0) {  // once per key/value head: the non-mask rows go to their cache slots
                    const bool is_mask = kv_info[it] & 1;
                    const int slot = kv_slot[it];
                    const bool to_cache = !is_mask && slot >= 0 && slot < a.capacity;
                    if (!is_mask && !to_cache && i == 0 && h == 0) atomicAdd(a.faults, 1);
                    if (to_cache) {
                        bool bad = false;
                        const size_t run = kv_run_offset<PAGED>(a.paging, b, kvh, Hkv, a.capacity, DH, slot / kAttnKeys, &bad);
                        if (bad && i == 0) atomicAdd(a.faults, 1);
                        uint16_t* kc = a.kc_w + run + (size_t)(slot % kAttnKeys) * DH + i;
                        *(u32x2*)kc = kav;
                        *(u32x2*)(kc + half) = kbv;
                        uint16_t* vc = a.vc_w + run + (size_t)i * kAttnKeys + (slot % kAttnKeys);
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            vc[e * kAttnKeys] = va[e];
                            vc[(e + half) * kAttnKeys] = vb[e];
                        }
                    }
                }
            }
            // rows behind the block in its last chunk: cleared (a zero weight must not meet a stale non-finite value)
            const int pad_rows = n_blk * kAttnKeys - L;
            for (int u = threadIdx.x; u < pad_rows * (DH / 8); u += NTH) {
                const int r = L + u / (DH / 8), c = (u % (DH / 8)) * 8;
                *(u32x4*)(k_lds + r * KROW + c) = u32x4{0, 0, 0, 0};
            }
            for (int u = threadIdx.x; u < pad_rows * DH; u += NTH) {
                const int r = L + u / DH, d = u % DH;
                v_lds[((r / kAttnKeys) * DH + d) * VROW + (r % kAttnKeys)] = 0;
            }
        }
    }
    if (FUSE) {
        if (pre0) SPACE_ATTN_LOAD_V(av0, vb0_);
        if ((int)threadIdx.x < L) s_info[threadIdx.x] = own_info;
    } else {
        for (int i = threadIdx.x; i < L; i += WV * 64) s_info[i] = a.info[i];
    }
    __syncthreads();

    // (where the pipelined loop only meets cache chunks, which need no row facts, these are fetched behind
    // it: three registers the loop of the variant with three row tiles does not have)
    int my_row[TQ], my_info[TQ];
    auto row_facts = [&]() {
#pragma unroll
        for (int t = 0; t < TQ; ++t) {
            my_row[t] = r0 + 16 * t + c16;
            my_info[t] = s_info[min(my_row[t], L - 1)];
        }
    };
    if (!kLoopCacheOnly) row_facts();
    f32x4 o[DT][TQ];
    float m_w[TQ], l_w[TQ];  // running max (log2 domain) and sum of this wave's chunks
#pragma unroll
    for (int t = 0; t < TQ; ++t) {
        m_w[t] = -INFINITY;
        l_w[t] = 0.f;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) o[dt][t] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

// AFTER_PV runs at the end, when the value operands are free: the place where the values of the next
// chunk are requested into the same registers.
#define SPACE_ATTN_COMPUTE2(AK, AV, C, KEND, BLK, AFTER_PV)                                                 \
    do {                                                                                                    \
        /* Q is re-read from LDS for every chunk: keeping its 24 operand tiles in registers spills */      \
        asm volatile("" ::: "memory");                                                                      \
        f32x4 sc[2][TQ];                                                                                    \
        _Pragma("unroll") for (int tk = 0; tk < 2; ++tk) _Pragma("unroll") for (int t = 0; t < TQ; ++t)     \
            sc[tk][t] = f32x4{0.f, 0.f, 0.f, 0.f};                                                          \
        _Pragma("unroll") for (int t = 0; t < TQ; ++t) _Pragma("unroll") for (int ds = 0; ds < DS; ++ds) {  \
            const u32x4 qh_ = smem[((0 * TQ + t) * DS + ds) * 64 + lane];                                   \
            const u32x4 ql_ = smem[((1 * TQ + t) * DS + ds) * 64 + lane];                                   \
            _Pragma("unroll") for (int tk = 0; tk < 2; ++tk) {                                              \
                sc[tk][t] = mfma16(AK[tk][ds], qh_, sc[tk][t]);                                             \
                sc[tk][t] = mfma16(AK[tk][ds], ql_, sc[tk][t]);                                             \
            }                                                                                               \
        }                                                                                                   \
        /* a cache chunk that lies wholly below the length needs no masking at all */                      \
        const bool full_ = !BLK && (C + kAttnKeys <= KEND);                                                 \
        int kinfo[8] = {0, 0, 0, 0, 0, 0, 0, 0};                                                            \
        if (BLK) {                                                                                          \
            _Pragma("unroll") for (int j = 0; j < 8; ++j) kinfo[j] = s_info[min(C + 8 * g4 + j, L - 1)];    \
        }                                                                                                   \
        _Pragma("unroll") for (int t = 0; t < TQ; ++t) {                                                    \
            float val[8];                                                                                   \
            float cm = -INFINITY;                                                                           \
            if (full_) {                                                                                    \
                _Pragma("unroll") for (int j = 0; j < 8; ++j) {                                             \
                    val[j] = sc[j >> 2][t][j & 3] * scale_log2e;                                            \
                    cm = fmaxf(cm, val[j]);                                                                 \
                }                                                                                           \
            } else {                                                                                        \
                _Pragma("unroll") for (int j = 0; j < 8; ++j) {                                             \
                    const int key = C + 8 * g4 + j;                                                         \
                    const bool key_mask = kinfo[j] & 1;                                                     \
                    const bool same = (my_info[t] & 1) & ((my_info[t] >> 1) == (kinfo[j] >> 1));            \
                    const bool vis = (key <= my_row[t]) & (!key_mask | same);                               \
                    const bool ok = (key < KEND) & (!BLK | vis);                                            \
                    val[j] = ok ? sc[j >> 2][t][j & 3] * scale_log2e : -INFINITY;                           \
                    cm = fmaxf(cm, val[j]);                                                                 \
                }                                                                                           \
            }                                                                                               \
            cm = row_groups_max(cm);                                                                        \
            const float m_new = fmaxf(m_w[t], cm);                                                          \
            const float m_use = (m_new == -INFINITY) ? 0.f : m_new;                                         \
            const float alpha = __builtin_amdgcn_exp2f(m_w[t] - m_use);                                     \
            m_w[t] = m_new;                                                                                 \
            float psum = 0.f;                                                                               \
            uint32_t hi[8], lo[8];                                                                          \
            _Pragma("unroll") for (int j = 0; j < 8; ++j) {                                                 \
                const float p = __builtin_amdgcn_exp2f(val[j] - m_use);                                     \
                psum += p;                                                                                  \
                const uint16_t ph = f2bf(p);                                                                \
                hi[j] = ph;                                                                                 \
                lo[j] = f2bf(p - bf2f(ph));                                                                 \
            }                                                                                               \
            l_w[t] = l_w[t] * alpha + psum; /* this lane's 8 keys: the 4 lane groups of a row are added up once, at the end */ \
            const u32x4 p_hi = {hi[0] | (hi[1] << 16), hi[2] | (hi[3] << 16), hi[4] | (hi[5] << 16),        \
                                hi[6] | (hi[7] << 16)};                                                     \
            const u32x4 p_lo = {lo[0] | (lo[1] << 16), lo[2] | (lo[3] << 16), lo[4] | (lo[5] << 16),        \
                                lo[6] | (lo[7] << 16)};                                                     \
            if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) { /* the running max moved in some row */  \
                _Pragma("unroll") for (int dt = 0; dt < DT; ++dt) o[dt][t] *= alpha;                        \
            }                                                                                               \
            _Pragma("unroll") for (int dt = 0; dt < DT; ++dt) {                                             \
                o[dt][t] = mfma16(AV[dt], p_hi, o[dt][t]);                                                  \
                o[dt][t] = mfma16(AV[dt], p_lo, o[dt][t]);                                                  \
            }                                                                                               \
        }                                                                                                   \
        AFTER_PV;                                                                                           \
    } while (0)
#define SPACE_ATTN_COMPUTE(AK, AV, C, KEND, BLK) SPACE_ATTN_COMPUTE2(AK, AV, C, KEND, BLK, (void)0)

    // Software pipeline over this wave's chunks: the keys of the next chunk are requested before the current
    // one is computed (two key buffers), the values of the next chunk as soon as the current ones have
    // been used, into the same registers (one value buffer: with two the kernel does not fit 256
    // registers, and the compiler then copies operands to and from the accumulation registers for every
    // MFMA).  av0 is that buffer.
    {
        const uint16_t *nk, *nv;
        while (chunk < n_chunks) {
            SPACE_ATTN_PREP(nk, nv, c_1, kend_1, blk_1, chunk + chunk_step);
            SPACE_ATTN_LOAD_K(ak1, nk);
            SPACE_ATTN_COMPUTE2(ak0, av0, c_0, kend_0, blk_0, SPACE_ATTN_LOAD_V(av0, nv));
            chunk += chunk_step;
            if (chunk >= n_chunks) break;
            SPACE_ATTN_PREP(nk, nv, c_0, kend_0, blk_0, chunk + chunk_step);
            SPACE_ATTN_LOAD_K(ak0, nk);
            SPACE_ATTN_COMPUTE2(ak1, av0, c_1, kend_1, blk_1, SPACE_ATTN_LOAD_V(av0, nv));
            chunk += chunk_step;
        }
    }
    if (kLoopCacheOnly) row_facts();
    if (FUSE && blk_wg) {  // the block's own chunks out of LDS, one per wave
        for (int cb = wave; cb < n_blk; cb += WV) {
            const int kr = cb * kAttnKeys + 8 * (c16 >> 2) + (c16 & 3);
#pragma unroll
            for (int tk = 0; tk < 2; ++tk)
#pragma unroll
                for (int ds = 0; ds < DS; ++ds) ak0[tk][ds] = *(const u32x4*)(k_lds + (kr + 4 * tk) * KROW + 8 * g4 + 32 * ds);
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) av0[dt] = *(const u32x4*)(v_lds + (cb * DH + 16 * dt + c16) * VROW + 8 * g4);
            c_0 = cb * kAttnKeys;
            kend_0 = L;
            blk_0 = true;
            SPACE_ATTN_COMPUTE(ak0, av0, c_0, kend_0, blk_0);
        }
    }

    // merge of the waves: common max per row, rescale, add in wave order
#pragma unroll
    for (int t = 0; t < TQ; ++t) l_w[t] = row_groups_sum(l_w[t]);  // the 4 lane groups of a row, once
    if (g4 == 0) {
#pragma unroll
        for (int t = 0; t < TQ; ++t) {
            m_sh[wave][16 * t + c16] = m_w[t];
            l_sh[wave][16 * t + c16] = l_w[t];
        }
    }
    __syncthreads();
    float m_all[TQ], l_all[TQ];
#pragma unroll
    for (int t = 0; t < TQ; ++t) {
        float mx = -INFINITY;
        for (int w = 0; w < WV; ++w) mx = fmaxf(mx, m_sh[w][16 * t + c16]);
        const float m_use = (mx == -INFINITY) ? 0.f : mx;
        float ls = 0.f;
        for (int w = 0; w < WV; ++w) ls += l_sh[w][16 * t + c16] * exp2f(m_sh[w][16 * t + c16] - m_use);
        m_all[t] = mx;
        l_all[t] = ls;
        const float scale = exp2f(m_w[t] - m_use);  // 0 for a wave without visible keys
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) o[dt][t] *= scale;
    }
#pragma unroll
    for (int p0 = 0; p0 < DT; p0 += kPass) {
#pragma unroll
        for (int ps = 0; ps < kPass; ++ps)
#pragma unroll
            for (int t = 0; t < TQ; ++t) red[((wave * kPass + ps) * TQ + t) * 64 + lane] = o[p0 + ps][t];
        __syncthreads();
        if (wave < kPass) {  // wave w adds up slice p0 + w
            const int dt = p0 + wave;
#pragma unroll
            for (int t = 0; t < TQ; ++t) {
                f32x4 sum = red[((0 * kPass + wave) * TQ + t) * 64 + lane];
                for (int w = 1; w < WV; ++w) sum += red[((w * kPass + wave) * TQ + t) * 64 + lane];
                const int tok = my_row[t];
                if (tok >= L) continue;
                if (n_wg == 1) {
                    // the only workgroup of this (sequence, head, query group): normalise and write the
                    // operand planes of the output projection right here (same arithmetic as the merge
                    // kernel does for a single partial, which is then not launched)
                    const float wgt = l_all[t] > 0.f ? 1.0f / l_all[t] : 0.f;
                    uint32_t hi[4], lo[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float v = wgt * sum[e];
                        const uint16_t hv = f2bf(v);
                        hi[e] = hv;
                        lo[e] = f2bf(v - bf2f(hv));
                    }
                    const int col = h * DH + 16 * dt + 4 * g4;
                    *(u32x2*)(a.out + xt_index(b * L + tok, col, a.out_shape, 0)) = u32x2{hi[0] | (hi[1] << 16), hi[2] | (hi[3] << 16)};
                    *(u32x2*)(a.out + xt_index(b * L + tok, col, a.out_shape, 1)) = u32x2{lo[0] | (lo[1] << 16), lo[2] | (lo[3] << 16)};
                } else {
                    const size_t base = (bh * n_wg + wg) * L + tok;
                    *(f32x4*)(a.o_part + base * DH + 16 * dt + 4 * g4) = sum;
                }
            }
        }
        __syncthreads();
    }
    if (n_wg > 1 && wave == 0 && g4 == 0) {
#pragma unroll
        for (int t = 0; t < TQ; ++t) {
            const int tok = my_row[t];
            if (tok < L) {
                const size_t base = (bh * n_wg + wg) * L + tok;
                a.ml_part[base * 2] = m_all[t];
                a.ml_part[base * 2 + 1] = l_all[t];
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
// rotary + K/V store + attention + normalisation in one kernel, one workgroup per
// (sequence, head, query tile)
// ------------------------------------------------------------------------------------------
// While the block has at most 48 rows and the context is short, cutting a head over the key axis
// costs more (a staging kernel in front, a merge kernel behind, three dependent launches) than it
// gains.  Here a workgroup of 8 waves owns 16 query rows of a head.  It sums the projection's
// split partials and rotates its Q rows (straight to LDS as operand planes) and the K/V rows its
// queries can see (rows up to the end of its tile, by causality), which go to a staging slice of
// its own and, for the non-mask rows of its tile, to their cache slots.  The waves then take the
// 32-key chunks round robin exactly as above, merge through LDS in wave order and write the
// normalised output as operand planes.  The first cache chunk of every wave is requested before
// the staging work so that both latencies overlap.

constexpr int kHeadWaves = 8;

template <int DH, bool PAGED>
__global__ __launch_bounds__(kHeadWaves * 64) void attn_head_kernel(HeadAttnLaunch a, float scale_log2e) {
    constexpr int DS = DH / 32, DT = DH / 16, W = kHeadWaves, NT = kHeadWaves * 64, TQ = 1;
    constexpr bool kLoopCacheOnly = true;  // the pipelined loop never meets one of the block's own chunks
    constexpr int half = DH / 2;
    const int lane = threadIdx.x & 63, c16 = lane & 15, g4 = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int h = blockIdx.x, b = blockIdx.y, qt = blockIdx.z, QT = gridDim.z;
    const int L = a.L, H = a.n_heads, Hkv = a.n_kv_heads, hd = H * DH;
    const int ld = (H + 2 * Hkv) * DH;              // row length of the projection's partial sums
    const int group = H / Hkv, kvh = h / group;     // grouped-query attention: key/value head of this query head
    const size_t bh = (size_t)b * H + h;
    const int r0 = 16 * qt;
    const int kv_rows = min(L, r0 + 16);  // block keys visible to this tile


    __shared__ u32x4 smem[2 * DS * 64];  // Q operand planes [plane][ds][lane]
    __shared__ f32x4 red[W * DT * 64];   // merge buffer [wave][slice][lane]
    __shared__ float m_sh[W][16], l_sh[W][16], linv_sh[16];
    __shared__ int s_info[16 * kMaxRowTiles];
    // The block's own keys and values never leave the CU: K row-major, V transposed in runs of 32 keys as
    // in the cache, both with padded rows (272 / 80 bytes) so that the operand reads below spread over
    // the LDS banks.
    constexpr int kStageRows = (kHeadAttnMaxRows + kAttnKeys - 1) / kAttnKeys * kAttnKeys;
    constexpr int KROW = DH + 8, VROW = kAttnKeys + 8;
    __shared__ __attribute__((aligned(16))) uint16_t k_lds[kStageRows * KROW];
    __shared__ __attribute__((aligned(16))) uint16_t v_lds[kStageRows / kAttnKeys * DH * VROW];

    const uint16_t* kc_base = a.kc;  // + cache_off(chunk): contiguous run or page of this (sequence, head)
    const uint16_t* vc_base = a.vc;
    auto cache_off = [&](int ch) -> size_t { return kv_run_offset<PAGED>(a.paging, b, kvh, Hkv, a.capacity, DH, ch); };
    const uint16_t* kb_base = a.kc;  // the shared load macro wants block pointers; block chunks are read from LDS below
    const uint16_t* vb_base = a.vc;
    (void)bh; (void)QT;

    u32x4 ak0[2][DS], av0[DT], ak1[2][DS], av1[DT];
    int c_0 = 0, kend_0 = 1, c_1 = 0, kend_1 = 1;
    bool blk_0 = false, blk_1 = false;
    SPACE_ATTN_LANE_OFFSETS
    int chunk = wave;
    int len, n_cache, n_chunks;
    bool pre0, pre1;

    {
        // Staging work in items of 4 rotary pairs (columns i..i+3 and i+half..i+half+3 of one row):
        // 16 * (DH/8) Q items of this tile, then kv_rows * (DH/8) K/V items.  All partial sums of an
        // item are requested before any is used; a thread has at most one Q item and two K/V items.
        constexpr int IPR = half / 4;  // items per row
        typedef __attribute__((ext_vector_type(4))) float f4;
        uint16_t* q_lds = (uint16_t*)smem;
        const size_t ss = a.split_stride;
        const int tid = threadIdx.x;
        // ---- loads
        const bool has_q = tid < 16 * IPR;
        const int q_rr = tid / IPR, q_i = (tid % IPR) * 4, q_r = r0 + q_rr;
        const bool q_real = has_q && q_r < L;
        // Every load below is unconditional (rows past the end are clamped to a real row and their values
        // dropped) and, for the usual 1 or 2 partial sums, none is consumed before all are requested:
        // loads inside branches that also use them cost a memory round trip per branch, which is what
        // this prologue spent most of its time on.
        f4 qs0, qs1, q_c, q_s, ks0[2], ks1[2], vs0[2], vs1[2], kc_c[2], kc_s[2];
        int kv_r[2], kv_i[2], kv_info[2], kv_slot[2];
        bool kv_on[2];
        const float* kvb[2];
        const int q_row = b * L + min(q_r, L - 1);
        const float* qb = a.qkv + (size_t)q_row * ld + h * DH + q_i;
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const int u = tid + it * NT;
            kv_on[it] = u < kv_rows * IPR;
            kv_r[it] = min(u / IPR, kv_rows - 1);
            kv_i[it] = (u % IPR) * 4;
            kvb[it] = a.qkv + (size_t)(b * L + kv_r[it]) * ld + hd + kvh * DH + kv_i[it];
        }
        auto sums = [&](auto S_) {
            constexpr int S = decltype(S_)::value;
            f4 tq0[S], tq1[S], tk0[2][S], tk1[2][S], tv0[2][S], tv1[2][S];
#pragma unroll
            for (int sp = 0; sp < S; ++sp) {
                tq0[sp] = *(const f4*)(qb + sp * ss);
                tq1[sp] = *(const f4*)(qb + sp * ss + half);
            }
#pragma unroll
            for (int it = 0; it < 2; ++it)
#pragma unroll
                for (int sp = 0; sp < S; ++sp) {
                    tk0[it][sp] = *(const f4*)(kvb[it] + sp * ss);
                    tk1[it][sp] = *(const f4*)(kvb[it] + sp * ss + half);
                    tv0[it][sp] = *(const f4*)(kvb[it] + sp * ss + Hkv * DH);
                    tv1[it][sp] = *(const f4*)(kvb[it] + sp * ss + Hkv * DH + half);
                }
            const f4 z = {0.f, 0.f, 0.f, 0.f};
            qs0 = qs1 = z;
#pragma unroll
            for (int sp = 0; sp < S; ++sp) { qs0 += tq0[sp]; qs1 += tq1[sp]; }
#pragma unroll
            for (int it = 0; it < 2; ++it) {
                ks0[it] = ks1[it] = vs0[it] = vs1[it] = z;
#pragma unroll
                for (int sp = 0; sp < S; ++sp) {
                    ks0[it] += tk0[it][sp]; ks1[it] += tk1[it][sp];
                    vs0[it] += tv0[it][sp]; vs1[it] += tv1[it][sp];
                }
            }
        };
        // rotary factors and row facts first: they are consumed last
        const int info_own = a.info[min(tid, L - 1)];  // L <= 48 rows: one per thread, for the LDS copy below
        q_c = *(const f4*)(a.cos_t + (size_t)q_row * half + q_i);
        q_s = *(const f4*)(a.sin_t + (size_t)q_row * half + q_i);
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const int row = b * L + kv_r[it];
            kc_c[it] = *(const f4*)(a.cos_t + (size_t)row * half + kv_i[it]);
            kc_s[it] = *(const f4*)(a.sin_t + (size_t)row * half + kv_i[it]);
            kv_info[it] = a.info[kv_r[it]];
            kv_slot[it] = a.pos[row];
        }
        if (a.splits == 1) {
            sums(std::integral_constant<int, 1>{});
        } else if (a.splits == 2) {
            sums(std::integral_constant<int, 2>{});
        } else {  // more partial sums than registers for all of them at once: one after the other
            const f4 z = {0.f, 0.f, 0.f, 0.f};
            qs0 = qs1 = z;
            for (int sp = 0; sp < a.splits; ++sp) {
                qs0 += *(const f4*)(qb + sp * ss);
                qs1 += *(const f4*)(qb + sp * ss + half);
            }
#pragma unroll
            for (int it = 0; it < 2; ++it) {
                ks0[it] = ks1[it] = vs0[it] = vs1[it] = z;
                for (int sp = 0; sp < a.splits; ++sp) {
                    ks0[it] += *(const f4*)(kvb[it] + sp * ss);
                    ks1[it] += *(const f4*)(kvb[it] + sp * ss + half);
                    vs0[it] += *(const f4*)(kvb[it] + sp * ss + Hkv * DH);
                    vs1[it] += *(const f4*)(kvb[it] + sp * ss + Hkv * DH + half);
                }
            }
        }
        if (!q_real) {  // rows that pad the tile are zero
            qs0 = qs1 = f4{0.f, 0.f, 0.f, 0.f};
        }
        // ---- arithmetic: everything that was requested above is used up here, in registers
        // Q: rotary, hi + lo planes (rows that pad the tile are zero)
        u32x2 q_ah, q_bh, q_al, q_bl;
        {
            uint32_t ah[4], al[4], bh_[4], bl[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float ra = qs0[e] * q_c[e] - qs1[e] * q_s[e], rb = qs1[e] * q_c[e] + qs0[e] * q_s[e];
                const uint16_t ha = f2bf(ra), hb = f2bf(rb);
                ah[e] = ha; al[e] = f2bf(ra - bf2f(ha));
                bh_[e] = hb; bl[e] = f2bf(rb - bf2f(hb));
            }
            q_ah = u32x2{ah[0] | (ah[1] << 16), ah[2] | (ah[3] << 16)};
            q_bh = u32x2{bh_[0] | (bh_[1] << 16), bh_[2] | (bh_[3] << 16)};
            q_al = u32x2{al[0] | (al[1] << 16), al[2] | (al[3] << 16)};
            q_bl = u32x2{bl[0] | (bl[1] << 16), bl[2] | (bl[3] << 16)};
        }
        // K/V rows 0 .. kv_rows-1: rotary, and where this tile's own non-mask rows go in the cache
        u32x2 kav[2], kbv[2], vav[2], vbv[2];
        bool to_cache[2];
        size_t kc_off[2], vc_off[2];
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const int r = kv_r[it], i = kv_i[it];
            uint32_t ka[4], kb[4], va[4], vb[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                ka[e] = f2bf(ks0[it][e] * kc_c[it][e] - ks1[it][e] * kc_s[it][e]);
                kb[e] = f2bf(ks1[it][e] * kc_c[it][e] + ks0[it][e] * kc_s[it][e]);
                va[e] = f2bf(vs0[it][e]);
                vb[e] = f2bf(vs1[it][e]);
            }
            kav[it] = u32x2{ka[0] | (ka[1] << 16), ka[2] | (ka[3] << 16)};
            kbv[it] = u32x2{kb[0] | (kb[1] << 16), kb[2] | (kb[3] << 16)};
            vav[it] = u32x2{va[0] | (va[1] << 16), va[2] | (va[3] << 16)};
            vbv[it] = u32x2{vb[0] | (vb[1] << 16), vb[2] | (vb[3] << 16)};
            to_cache[it] = false;
            kc_off[it] = vc_off[it] = 0;
            if (kv_on[it] && r >= r0 && h % group == 0) {  // this tile's own rows also go to the cache (once per key/value head)
                const bool is_mask = kv_info[it] & 1;
                const int slot = kv_slot[it];
                to_cache[it] = !is_mask && slot >= 0 && slot < a.capacity;
                if (!is_mask && !to_cache[it] && i == 0 && h == 0) atomicAdd(a.faults, 1);
                if (to_cache[it]) {
                    bool bad = false;
                    const size_t run = kv_run_offset<PAGED>(a.paging, b, kvh, Hkv, a.capacity, DH, slot / kAttnKeys, &bad);
                    if (bad && i == 0) atomicAdd(a.faults, 1);
                    kc_off[it] = run + (size_t)(slot % kAttnKeys) * DH + i;
                    vc_off[it] = run + (size_t)i * kAttnKeys + (slot % kAttnKeys);
                }
            }
        }
        static_assert(kHeadAttnMaxRows <= NT, "one row fact per thread");
        if (tid < L) s_info[tid] = info_own;
        // ---- the first two cache chunks of this wave (the block's own chunks only exist after the staging
        // work), so that their latency and the staging's stores overlap.  Nothing below uses a value that
        // was requested before them: loads come back in order, and behind requests that sit in a branch the
        // compiler waits for all of them, so a use of an older load down there would wait for the chunks.
        // (Requested at the very start instead, the first chunk holds up the partial sums behind it -- loads
        // come back in order -- and the kernel takes as long.)
        __builtin_amdgcn_sched_barrier(0);
        len = min(max(a.kv_len[b], 0), a.capacity);
        n_cache = (len + kAttnKeys - 1) / kAttnKeys;
        n_chunks = n_cache;  // of the pipelined loop: the block's own chunks come from LDS afterwards
        pre0 = chunk < n_cache;
        pre1 = chunk + W < n_cache;
        if (pre0) SPACE_ATTN_LOAD(ak0, av0, c_0, kend_0, blk_0, chunk);
        if (pre1) SPACE_ATTN_LOAD(ak1, av1, c_1, kend_1, blk_1, chunk + W);
        __builtin_amdgcn_sched_barrier(0);
        // ---- stores
        // rows of the last block chunk that no query of this tile sees: cleared, so that a zero weight
        // never meets a stale non-finite value
        {
            const int pad_rows = (kv_rows + kAttnKeys - 1) / kAttnKeys * kAttnKeys - kv_rows;
            for (int u = tid; u < pad_rows * (DH / 8); u += NT) {
                const int r = kv_rows + u / (DH / 8), c = (u % (DH / 8)) * 8;
                *(u32x4*)(k_lds + r * KROW + c) = u32x4{0, 0, 0, 0};
            }
            for (int u = tid; u < pad_rows * DH; u += NT) {
                const int r = kv_rows + u / DH, d = u % DH;
                v_lds[((r / kAttnKeys) * DH + d) * VROW + (r % kAttnKeys)] = 0;
            }
        }
        if (has_q) {
            // element (plane, rr, col): (((plane*DS + col/32)*64 + rr + 16*((col%32)/8))*8 + col%8
            const int qa_i = (((q_i >> 5) * 64 + q_rr + 16 * ((q_i & 31) >> 3)) << 3) + (q_i & 7);
            const int qb_i = qa_i + (half >> 5) * 64 * 8;
            constexpr int lo_off = DS * 64 * 8;
            *(u32x2*)(q_lds + qa_i) = q_ah;
            *(u32x2*)(q_lds + qb_i) = q_bh;
            *(u32x2*)(q_lds + qa_i + lo_off) = q_al;
            *(u32x2*)(q_lds + qb_i + lo_off) = q_bl;
        }
        // K/V -> this workgroup's staging slice (+ the cache slots of its own tile)
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            if (!kv_on[it]) continue;
            const int r = kv_r[it], i = kv_i[it];
            uint16_t* ko = k_lds + r * KROW + i;
            *(u32x2*)ko = kav[it];
            *(u32x2*)(ko + half) = kbv[it];
            uint16_t* vo = v_lds + ((r / kAttnKeys) * DH + i) * VROW + (r % kAttnKeys);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                vo[e * VROW] = (uint16_t)(vav[it][e >> 1] >> (16 * (e & 1)));
                vo[(e + half) * VROW] = (uint16_t)(vbv[it][e >> 1] >> (16 * (e & 1)));
            }
            if (to_cache[it]) {
                uint16_t* kc = a.kc + kc_off[it];
                *(u32x2*)kc = kav[it];
                *(u32x2*)(kc + half) = kbv[it];
                uint16_t* vc = a.vc + vc_off[it];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    vc[e * kAttnKeys] = (uint16_t)(vav[it][e >> 1] >> (16 * (e & 1)));
                    vc[(e + half) * kAttnKeys] = (uint16_t)(vbv[it][e >> 1] >> (16 * (e & 1)));
                }
            }
        }
    }

    // the staging rows are read back below by other waves of this workgroup
    __syncthreads();


    int my_row[TQ], my_info[TQ];
    my_row[0] = r0 + c16;
    my_info[0] = s_info[min(my_row[0], L - 1)];
    f32x4 o[DT][TQ];
    float m_w[TQ], l_w[TQ];
    m_w[0] = -INFINITY;
    l_w[0] = 0.f;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) o[dt][0] = f32x4{0.f, 0.f, 0.f, 0.f};

    // cache chunks, two in flight: buffer 0 holds chunk, buffer 1 chunk + W (both were requested above)
    while (chunk < n_chunks) {
        SPACE_ATTN_COMPUTE(ak0, av0, c_0, kend_0, blk_0);
        SPACE_ATTN_LOAD(ak0, av0, c_0, kend_0, blk_0, chunk + 2 * W);
        chunk += W;
        if (chunk >= n_chunks) break;
        SPACE_ATTN_COMPUTE(ak1, av1, c_1, kend_1, blk_1);
        SPACE_ATTN_LOAD(ak1, av1, c_1, kend_1, blk_1, chunk + 2 * W);
        chunk += W;
    }
    // the block's own chunks, out of LDS: they continue the round robin behind the cache chunks, so the
    // waves with one cache chunk fewer take them
    {
        const int n_blk = (kv_rows + kAttnKeys - 1) / kAttnKeys;
        for (int cb = (wave - n_cache % W + W) % W; cb < n_blk; cb += W) {
            const int kr = cb * kAttnKeys + 8 * (c16 >> 2) + (c16 & 3);
#pragma unroll
            for (int tk = 0; tk < 2; ++tk)
#pragma unroll
                for (int ds = 0; ds < DS; ++ds) ak0[tk][ds] = *(const u32x4*)(k_lds + (kr + 4 * tk) * KROW + 8 * g4 + 32 * ds);
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) av0[dt] = *(const u32x4*)(v_lds + (cb * DH + 16 * dt + c16) * VROW + 8 * g4);
            c_0 = cb * kAttnKeys;
            kend_0 = L;
            blk_0 = true;
            SPACE_ATTN_COMPUTE(ak0, av0, c_0, kend_0, blk_0);
        }
    }


    l_w[0] = row_groups_sum(l_w[0]);  // the 4 lane groups of a row, once
    if (g4 == 0) {
        m_sh[wave][c16] = m_w[0];
        l_sh[wave][c16] = l_w[0];
    }
    __syncthreads();
    {
        float mx = -INFINITY;
        for (int w = 0; w < W; ++w) mx = fmaxf(mx, m_sh[w][c16]);
        const float m_use = (mx == -INFINITY) ? 0.f : mx;
        float ls = 0.f;
        for (int w = 0; w < W; ++w) ls += l_sh[w][c16] * exp2f(m_sh[w][c16] - m_use);
        if (wave == 0 && g4 == 0) linv_sh[c16] = ls > 0.f ? 1.0f / ls : 0.f;
        const float scale = exp2f(m_w[0] - m_use);  // 0 for a wave without visible keys
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) red[(wave * DT + dt) * 64 + lane] = o[dt][0] * scale;
    }
    __syncthreads();

    for (int dt = wave; dt < DT; dt += W) {  // wave w adds up slice w in wave order
        f32x4 sum = red[dt * 64 + lane];
        for (int w = 1; w < W; ++w) sum += red[(w * DT + dt) * 64 + lane];
        const int tok = r0 + c16;
        if (tok < L) {
            sum *= linv_sh[c16];
            const int row = b * L + tok, col = h * DH + 16 * dt + 4 * g4;
            uint32_t hi[4], lo[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint16_t hh = f2bf(sum[e]);
                hi[e] = hh;
                lo[e] = f2bf(sum[e] - bf2f(hh));
            }
            *(u32x2*)(a.out + xt_index(row, col, a.out_shape, 0)) = u32x2{hi[0] | (hi[1] << 16), hi[2] | (hi[3] << 16)};
            *(u32x2*)(a.out + xt_index(row, col, a.out_shape, 1)) = u32x2{lo[0] | (lo[1] << 16), lo[2] | (lo[3] << 16)};
        }
    }

}
#undef SPACE_ATTN_LANE_OFFSETS
#undef SPACE_ATTN_LOAD
#undef SPACE_ATTN_PREP
#undef SPACE_ATTN_LOAD_K
#undef SPACE_ATTN_LOAD_V
#undef SPACE_ATTN_COMPUTE2
#undef SPACE_ATTN_COMPUTE

hipError_t launch_head_attention(const HeadAttnLaunch& a, hipStream_t s) {
    if (a.L < 1 || a.L > kHeadAttnMaxRows || (a.capacity % kAttnKeys) || a.capacity < kAttnKeys ||
        (a.Lp % kAttnKeys) || a.Lp < a.L || a.splits < 1 || a.splits > 8 || a.out_shape.row_tiles < 1 ||
        a.n_kv_heads < 1 || a.n_heads % a.n_kv_heads)
        return hipErrorInvalidValue;
    const dim3 grid(a.n_heads, a.batch, ceil_div(a.L, 16)), block(kHeadWaves * 64);
    if (a.paging.table && (a.paging.table_stride * kAttnKeys != a.capacity || a.paging.n_pages < 1)) return hipErrorInvalidValue;
    const bool paged = a.paging.table != nullptr;
    if (a.head_dim == 128) {
        const float scale_log2e = (float)(1.4426950408889634 / sqrt(128.0));
        if (paged) hipLaunchKernelGGL((attn_head_kernel<128, true>), grid, block, 0, s, a, scale_log2e);
        else hipLaunchKernelGGL((attn_head_kernel<128, false>), grid, block, 0, s, a, scale_log2e);
    } else if (a.head_dim == 64) {
        const float scale_log2e = (float)(1.4426950408889634 / sqrt(64.0));
        if (paged) hipLaunchKernelGGL((attn_head_kernel<64, true>), grid, block, 0, s, a, scale_log2e);
        else hipLaunchKernelGGL((attn_head_kernel<64, false>), grid, block, 0, s, a, scale_log2e);
    } else {
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// merge of the per-workgroup (max, sum, O) triples; writes the operand planes of the output projection
__global__ void attn_combine_kernel(AttnLaunch a, int n_wg) {
    __shared__ float w_sh[64];  // weight of each partial, already divided by the total sum
    // heads on the fast grid axis: with a multiple of 8 heads all rows of a head go to one XCD, whose L2
    // then collects whole lines of the operand planes (8 consecutive rows share each of them)
    const int row = blockIdx.y, h = blockIdx.x, d = threadIdx.x;
    const int DH = a.head_dim, L = a.L, H = a.n_heads;
    const int b = row / L, r = row % L;
    const size_t bh = (size_t)b * H + h;
    if (d < 64) {  // one wave: statistics of up to 64 partials, one per lane
        float m = -INFINITY, l = 0.f;
        if (d < n_wg) {
            const size_t base = (bh * n_wg + d) * L + r;
            m = a.ml_part[base * 2];
            l = a.ml_part[base * 2 + 1];
        }
        float mx = m;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
        const float wgt = (m == -INFINITY) ? 0.f : exp2f(m - mx);
        float den = wgt * l;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) den += __shfl_xor(den, o, 64);
        w_sh[d] = den > 0.f ? wgt / den : 0.f;
    }
    __syncthreads();
    float num = 0.f;
#pragma unroll 8
    for (int s = 0; s < n_wg; ++s) {
        const float wgt = w_sh[s];
        const float v = a.o_part[((bh * n_wg + s) * L + r) * DH + d];
        num += wgt != 0.f ? wgt * v : 0.f;  // an empty partial may hold anything
    }
    xt_store(a.out, row, h * DH + d, a.out_shape, num);
}

// Workgroups along the key axis for `streams` (sequence, head, query group) triples: one chunk per
// wave while that keeps the grid at or under 256 workgroups, more rounds per wave beyond.  Two
// 4-wave workgroups fit a CU (at most 256 registers, under half its LDS), which is what lets the 512
// workgroups of a long block with two query groups run at once; cutting the keys finer than one workgroup per CU
// still loses (every workgroup stages the queries again): with a cap of 512, 13B at 2048 positions 26.8 ->
// 29.4 us per layer, a ragged batch of 8 at k = 5 88 -> 93 us.
int attention_workgroups(int len_bound, int L, int streams) {
    constexpr int waves = 4;
    const int chunks = ceil_div(len_bound, kAttnKeys) + ceil_div(L, kAttnKeys);
    int cap = 256 / (streams > 0 ? streams : 1);
    if (cap < 1) cap = 1;
    if (cap > 64) cap = 64;  // the merge pass handles one partial per lane
    const int want = ceil_div(chunks, waves);
    return want < cap ? want : cap;
}

template <int DH, bool PAGED>
static hipError_t launch_attention_dh(const AttnLaunch& a, hipStream_t s) {
    const float scale_log2e = (float)(1.4426950408889634 / sqrt((double)DH));
    const int tiles = ceil_div(a.L, 16);
    const int TQ = tiles >= 3 ? 3 : tiles;
    const int QG = ceil_div(tiles, TQ);
    const dim3 grid(a.n_wg, a.n_heads, a.batch * QG), block(4 * 64);
    if (a.qkv) {  // rotary and K/V staging inside the kernel: one query group, at most 48 rows
        if (QG != 1 || a.L > kHeadAttnMaxRows || a.splits < 1 || !a.cos_t || !a.sin_t || !a.pos || !a.kc_w || !a.vc_w || !a.faults)
            return hipErrorInvalidValue;
        switch (TQ) {
            case 1: hipLaunchKernelGGL((attn_sar_kernel<DH, 1, PAGED, true, 4>), grid, block, 0, s, a, scale_log2e); break;
            case 2: hipLaunchKernelGGL((attn_sar_kernel<DH, 2, PAGED, true, 4>), grid, block, 0, s, a, scale_log2e); break;
            default: hipLaunchKernelGGL((attn_sar_kernel<DH, 3, PAGED, true, 4>), grid, block, 0, s, a, scale_log2e); break;
        }
    } else {
        switch (TQ) {
            case 1: hipLaunchKernelGGL((attn_sar_kernel<DH, 1, PAGED, false, 4>), grid, block, 0, s, a, scale_log2e); break;
            case 2: hipLaunchKernelGGL((attn_sar_kernel<DH, 2, PAGED, false, 4>), grid, block, 0, s, a, scale_log2e); break;
            default: hipLaunchKernelGGL((attn_sar_kernel<DH, 3, PAGED, false, 4>), grid, block, 0, s, a, scale_log2e); break;
        }
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || a.n_wg == 1) return e;  // a single workgroup along the keys writes the output itself
    hipLaunchKernelGGL(attn_combine_kernel, dim3(a.n_heads, a.batch * a.L), dim3(DH), 0, s, a, a.n_wg);
    return hipGetLastError();
}

hipError_t launch_attention(const AttnLaunch& a, hipStream_t s) {
    if (a.L < 1 || a.L > kMaxBlockRows || (a.capacity % kAttnKeys) || (a.Lp % kAttnKeys) || a.n_wg < 1 ||
        a.n_wg > 64 || a.n_kv_heads < 1 || a.n_heads % a.n_kv_heads)
        return hipErrorInvalidValue;
    if (a.paging.table && (a.paging.table_stride * kAttnKeys != a.capacity || a.paging.n_pages < 1)) return hipErrorInvalidValue;
    const bool paged = a.paging.table != nullptr;
    if (a.head_dim == 128) return paged ? launch_attention_dh<128, true>(a, s) : launch_attention_dh<128, false>(a, s);
    if (a.head_dim == 64) return paged ? launch_attention_dh<64, true>(a, s) : launch_attention_dh<64, false>(a, s);
    return hipErrorInvalidValue;
}

// ------------------------------------------------------------------------------------------
// final argmax over the per-workgroup partials + greedy verification (Algorithm 1)
// ------------------------------------------------------------------------------------------
// accepted = longest prefix of candidates with c_{i+1} == argmax(row of c_i) (row of x_l for i = 0);
// the extra token is the argmax of the last accepted row; the new candidates are the argmax of
// the mask rows that follow it; the next block is assembled on the device so that the host
// never has to sit between two steps.

__global__ __launch_bounds__(1024) void verify_kernel(VerifyLaunch v) {
    constexpr int kRows = 16 * kMaxRowTiles;
    __shared__ int s_arg[kRows], s_tok[kRows], s_real[kRows], s_nmask[kRows], s_next[kRows];
    __shared__ int s_bonus, s_last, s_nm;
    const int b = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
    const int L = v.lay.L, G = v.lay.G;
    // everything the scan needs goes to LDS with independent loads
    // thread 0 needs the emit position and the finished flag at the very end: asked for now
    int emit_n = 0, emit_fin = 0;
    if (threadIdx.x == 0 && v.emit && v.emit_len) {
        emit_n = v.emit_len[b];
        emit_fin = v.finished ? v.finished[b] : 0;
    }
    for (int i = threadIdx.x; i < L; i += blockDim.x) s_tok[i] = v.tokens[(size_t)b * L + i];
    for (int i = threadIdx.x; i < G; i += blockDim.x) {
        s_real[i] = v.lay.real_row[i];
        s_nmask[i] = v.lay.n_mask[i];
    }
    if (v.next_tokens)
        for (int i = threadIdx.x; i < v.next.L; i += blockDim.x) s_next[i] = v.next.info[i];
    for (int r = wave; r < L; r += nwaves) {
        const size_t row = (size_t)b * L + r;
        float best = -INFINITY;
        int bi = INT_MAX;
        for (int g = lane; g < v.n_groups_used; g += 64) {
            const float val = v.arg_val[row * v.arg_groups + g];
            const int idx = v.arg_idx[row * v.arg_groups + g];
            if (val > best || (val == best && idx < bi)) { best = val; bi = idx; }
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            const float ov = __shfl_xor(best, o, 64);
            const int oi = __shfl_xor(bi, o, 64);
            if (ov > best || (ov == best && oi < bi)) { best = ov; bi = oi; }
        }
        if (lane == 0) {
            s_arg[r] = bi;
            v.argmax_ws[row] = bi;
            if (v.argmax) v.argmax[row] = bi;
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int acc = 0;
        while (acc < G - 1 && s_tok[s_real[acc + 1]] == s_arg[s_real[acc]]) ++acc;
        const int last = s_real[acc];
        s_last = last;
        s_bonus = s_arg[last];
        s_nm = s_nmask[acc];
        v.accepted_ws[b] = acc;
        if (v.accepted_len) v.accepted_len[b] = acc;
        if (v.bonus) v.bonus[b] = s_arg[last];
        if (v.emit && v.emit_len) {
            // the accepted candidates and the extra token are the argmax of rows real[0..acc]; an end-of-
            // sequence token cuts the output in front of it and ends the sequence (Algorithm 1, EOS check)
            int n = emit_n;
            bool fin = emit_fin != 0;
            for (int i = 0; i <= acc && !fin; ++i) {
                const int t = s_arg[s_real[i]];
                if (v.eos_id >= 0 && t == v.eos_id) { fin = true; break; }
                if (n < v.emit_cap) v.emit[(size_t)b * v.emit_cap + n++] = t;
            }
            v.emit_len[b] = n;
            if (v.finished) v.finished[b] = fin;
        }
    }
    __syncthreads();
    const int last = s_last, nm = s_nm, bonus = s_bonus;
    if (v.new_cands)
        for (int j = threadIdx.x; j < v.max_cands; j += blockDim.x)
            v.new_cands[(size_t)b * v.max_cands + j] = j < nm ? s_arg[last + 1 + j] : -1;
    if (v.next_tokens)
        for (int r = threadIdx.x; r < v.next.L; r += blockDim.x) {
            const int inf = s_next[r], g = inf >> 1;
            int tok;
            if (inf & 1) tok = v.mask_id;
            else if (g == 0) tok = bonus;
            else tok = (g - 1 < nm) ? s_arg[last + g] : 0;
            v.next_tokens[(size_t)b * v.next.L + r] = tok;
        }
}

hipError_t launch_verify(const VerifyLaunch& v, hipStream_t s) {
    // the kernel keeps the rows of this block and of the next one in LDS arrays of 96 entries
    if (v.lay.L < 1 || v.lay.L > 16 * kMaxRowTiles || v.lay.G < 1 || v.lay.G > v.lay.L ||
        (v.next_tokens && v.next.L > 16 * kMaxRowTiles))
        return hipErrorInvalidValue;
    hipLaunchKernelGGL(verify_kernel, dim3(v.batch), dim3(1024), 0, s, v);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// verification by rejection sampling (Algorithm 1 as printed; appendix "Random Sampling")
// ------------------------------------------------------------------------------------------
// Kernel 1, one workgroup per block row: the top_k largest logits in descending order (ties: lowest
// id), softmax over them, the shortest prefix whose mass reaches top_p, renormalised.  The j-th
// largest is the maximum of the elements that come after the (j-1)-th in that order, so no
// element is ever modified; a thread keeps its first 32 elements in registers.  Sums run
// sequentially in descending order in one thread: the result does not depend on the launch shape.

__device__ __forceinline__ bool sample_after(float v, int i, float pv, int pi) {  // (v, i) comes after (pv, pi)
    return v < pv || (v == pv && i > pi);
}
__device__ __forceinline__ bool sample_before(float v, int i, float bv, int bi) {
    return v > bv || (v == bv && i < bi);
}

__global__ __launch_bounds__(1024) void topk_warp_kernel(SampleLaunch a) {
    __shared__ float s_v[16];
    __shared__ int s_i[16];
    __shared__ float top_v[kMaxTopK], top_e[kMaxTopK];
    __shared__ int top_i[kMaxTopK];
    const int r = blockIdx.x, b = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const size_t row = (size_t)b * a.lay.L + r;
    const float* __restrict__ x = a.logits + row * a.vocab;
    const int V = a.vocab;
    constexpr int NC = 32;
    float cache[NC];
#pragma unroll
    for (int j = 0; j < NC; ++j) {
        const int i = tid + j * 1024;
        cache[j] = i < V ? x[i] : -INFINITY;
    }
    const int K = min(a.top_k, V);
    // Best and second best element of this thread.  After a round only the winner's owner moves on: to
    // its second best if it still knows it, else (a thread that wins a third time, rare) by a rescan.
    float mv = -INFINITY, nv = -INFINITY;
    int mi = INT_MAX, ni = INT_MAX;
    bool second_known = true;
#pragma unroll
    for (int j = 0; j < NC; ++j) {
        const int i = tid + j * 1024;
        const float v = cache[j];
        if (i < V) {
            if (sample_before(v, i, mv, mi)) { nv = mv; ni = mi; mv = v; mi = i; }
            else if (sample_before(v, i, nv, ni)) { nv = v; ni = i; }
        }
    }
    for (int i = tid + NC * 1024; i < V; i += 1024) {
        const float v = x[i];
        if (sample_before(v, i, mv, mi)) { nv = mv; ni = mi; mv = v; mi = i; }
        else if (sample_before(v, i, nv, ni)) { nv = v; ni = i; }
    }
    for (int k = 0; k < K; ++k) {
        float bv = mv;
        int bi = mi;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            const float ov = __shfl_xor(bv, o, 64);
            const int oi = __shfl_xor(bi, o, 64);
            if (sample_before(ov, oi, bv, bi)) { bv = ov; bi = oi; }
        }
        if (lane == 0) { s_v[wave] = bv; s_i[wave] = bi; }
        __syncthreads();
        bv = s_v[0]; bi = s_i[0];
        for (int w = 1; w < 16; ++w)
            if (sample_before(s_v[w], s_i[w], bv, bi)) { bv = s_v[w]; bi = s_i[w]; }
        if (tid == 0) { top_v[k] = bv; top_i[k] = bi; }
        if (mi == bi && second_known) {
            mv = nv; mi = ni;
            second_known = false;
        } else if (mi == bi) {  // everything of mine that is left comes after the winner in the order
            mv = -INFINITY;
            mi = INT_MAX;
#pragma unroll
            for (int j = 0; j < NC; ++j) {
                const int i = tid + j * 1024;
                const float v = cache[j];
                if (i < V && sample_after(v, i, bv, bi) && sample_before(v, i, mv, mi)) { mv = v; mi = i; }
            }
            for (int i = tid + NC * 1024; i < V; i += 1024) {
                const float v = x[i];
                if (sample_after(v, i, bv, bi) && sample_before(v, i, mv, mi)) { mv = v; mi = i; }
            }
        }
        __syncthreads();
    }
    if (tid == 0) {
        float* e = top_e;  // LDS: a per-thread array would live in scratch memory, a round trip per access
        float total = 0.f;
        for (int j = 0; j < K; ++j) {
            e[j] = expf(top_v[j] - top_v[0]);
            total += e[j];
        }
        int keep = K;
        float run = 0.f;
        for (int j = 0; j < K; ++j) {
            e[j] = e[j] / total;
            run += e[j];
            if (run >= a.top_p) { keep = j + 1; break; }
        }
        float mass = 0.f;
        for (int j = 0; j < keep; ++j) mass += e[j];
        for (int j = 0; j < keep; ++j) {
            a.row_ids[row * kMaxTopK + j] = top_i[j];
            a.row_probs[row * kMaxTopK + j] = e[j] / mass;
        }
        a.row_n[row] = keep;
    }
}

// Kernel 2, one workgroup per sequence: thread 0 walks lines 6-22 of Algorithm 1 over the lists.
__device__ float sample_prob_of(const int* ids, const float* probs, int n, int token) {
    for (int j = 0; j < n; ++j)
        if (ids[j] == token) return probs[j];
    return 0.f;
}
__device__ int sample_draw(const int* ids, const float* probs, int n, float u, float* p_out) {
    float run = 0.f;
    for (int j = 0; j < n; ++j) {
        run += probs[j];
        if (u < run) { *p_out = probs[j]; return ids[j]; }
    }
    *p_out = probs[n - 1];
    return ids[n - 1];
}

__global__ __launch_bounds__(256) void sample_verify_kernel(SampleLaunch v) {
    constexpr int kRows = 16 * kMaxRowTiles;
    __shared__ int s_extra, s_last, s_nm;
    __shared__ int s_new[kRows], s_tok[kRows], s_n[kRows], s_real[kRows], s_nmask[kRows];
    __shared__ float s_u[2 * kRows], s_pc[kRows], s_res[kMaxTopK];
    extern __shared__ int s_lists[];  // [L][top_k] ids, then [L][top_k] probabilities
    const int b = blockIdx.x;
    const int L = v.lay.L, G = v.lay.G, K = v.top_k;
    const int NU = G + v.max_cands;
    int* l_ids = s_lists;
    float* l_probs = (float*)(s_lists + L * K);
    // everything the walk needs goes to LDS with independent loads
    for (int i = threadIdx.x; i < L * K; i += blockDim.x) {
        const size_t row = (size_t)b * L + i / K;
        l_ids[i] = v.row_ids[row * kMaxTopK + i % K];
        l_probs[i] = v.row_probs[row * kMaxTopK + i % K];
    }
    for (int i = threadIdx.x; i < L; i += blockDim.x) {
        s_tok[i] = v.tokens[(size_t)b * L + i];
        s_n[i] = v.row_n[(size_t)b * L + i];
    }
    for (int i = threadIdx.x; i < G; i += blockDim.x) {
        s_real[i] = v.lay.real_row[i];
        s_nmask[i] = v.lay.n_mask[i];
    }
    for (int i = threadIdx.x; i < NU; i += blockDim.x) s_u[i] = v.uniforms[(size_t)b * NU + i];
    for (int i = threadIdx.x; i < v.max_cands; i += blockDim.x) s_pc[i] = v.p_c[(size_t)b * v.max_cands + i];
    __syncthreads();
    const float* u = s_u;
    if (threadIdx.x == 0) {
        int acc = 0, rejected = 0;
        int qrow = s_real[0];
        for (int i = 1; i < G; ++i) {
            const int c = s_tok[s_real[i]];
            const float q = sample_prob_of(l_ids + qrow * K, l_probs + qrow * K, s_n[qrow], c);
            const float ratio = q / s_pc[i - 1];
            if (v.ratios) v.ratios[(size_t)b * (G - 1) + (i - 1)] = ratio;
            if (u[i - 1] <= ratio) {
                ++acc;
                qrow = s_real[i];
            } else {
                rejected = i;
                break;
            }
        }
        if (v.ratios)
            for (int i = (rejected ? rejected : G - 1) + 1; i < G; ++i) v.ratios[(size_t)b * (G - 1) + (i - 1)] = -1.f;
        // the extra token
        const int* q_ids = l_ids + qrow * K;
        const float* q_probs = l_probs + qrow * K;
        const int qn = s_n[qrow];
        float p_extra;
        float* res = s_res;
        bool use_res = false;
        if (v.residual && rejected && v.draft_ids && v.draft_probs) {
            const size_t d0 = ((size_t)b * v.max_cands + (rejected - 1)) * K;
            int dn = 0;
            while (dn < K && v.draft_ids[d0 + dn] >= 0) ++dn;
            float sum = 0.f;
            for (int j = 0; j < qn; ++j) {
                const float d = q_probs[j] - sample_prob_of(v.draft_ids + d0, v.draft_probs + d0, dn, q_ids[j]);
                res[j] = d > 0.f ? d : 0.f;
                sum += res[j];
            }
            if (sum > 0.f) {
                for (int j = 0; j < qn; ++j) res[j] = res[j] / sum;
                use_res = true;
            }
        }
        const int extra = sample_draw(q_ids, use_res ? res : q_probs, qn, u[G - 1], &p_extra);
        s_extra = extra; s_last = s_real[acc]; s_nm = s_nmask[acc];
        v.accepted_ws[b] = acc;
        v.accepted_len[b] = acc;
        v.extra[b] = extra;
        if (v.emit && v.emit_len) {
            int n = v.emit_len[b];
            bool fin = v.finished && v.finished[b] != 0;
            for (int i = 1; i <= acc + 1 && !fin; ++i) {  // accepted candidates, then the extra token
                const int t = i <= acc ? s_tok[s_real[i]] : extra;
                if (v.eos_id >= 0 && t == v.eos_id) { fin = true; break; }
                if (n < v.emit_cap) v.emit[(size_t)b * v.emit_cap + n++] = t;
            }
            v.emit_len[b] = n;
            if (v.finished) v.finished[b] = fin;
        }
    }
    __syncthreads();
    const int last = s_last, nm = s_nm;
    // the new candidates: thread j draws from the j-th mask row behind the last accepted row
    for (int j = threadIdx.x; j < v.max_cands; j += blockDim.x) {
        int t = -1;
        float pt = 0.f;
        const size_t o = ((size_t)b * v.max_cands + j) * K;
        const int row = last + 1 + j;
        const int n = j < nm ? s_n[row] : 0;
        if (j < nm) t = sample_draw(l_ids + row * K, l_probs + row * K, n, u[G + j], &pt);
        for (int q = 0; q < K; ++q) {
            if (v.new_ids) v.new_ids[o + q] = q < n ? l_ids[row * K + q] : -1;
            if (v.new_probs) v.new_probs[o + q] = q < n ? l_probs[row * K + q] : 0.f;
        }
        v.new_cands[(size_t)b * v.max_cands + j] = t;
        v.new_pc[(size_t)b * v.max_cands + j] = pt;
        s_new[j] = t;
    }
    __syncthreads();
    if (v.next_tokens)
        for (int r = threadIdx.x; r < v.next.L; r += blockDim.x) {
            const int inf = v.next.info[r], g = inf >> 1;
            int tok;
            if (inf & 1) tok = v.mask_id;
            else if (g == 0) tok = s_extra;
            else tok = (g - 1 < nm) ? s_new[g - 1] : 0;
            v.next_tokens[(size_t)b * v.next.L + r] = tok;
        }
}

hipError_t launch_sample_verify(const SampleLaunch& v, hipStream_t s) {
    if (v.top_k < 1 || v.top_k > kMaxTopK || !(v.top_p > 0.f) || v.top_p > 1.f || v.lay.L < 1 || v.lay.G < 1 ||
        v.max_cands < 1 || v.max_cands > 16 * kMaxRowTiles)
        return hipErrorInvalidValue;
    // both kernels keep per-row facts in LDS arrays of 96 entries (uniforms: 192): check before either is enqueued
    if (v.lay.L > 16 * kMaxRowTiles || v.lay.G + v.max_cands > 2 * 16 * kMaxRowTiles) return hipErrorInvalidValue;
    hipLaunchKernelGGL(topk_warp_kernel, dim3(v.lay.L, v.batch), dim3(1024), 0, s, v);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const size_t lds = (size_t)v.lay.L * v.top_k * 8;  // at most 96 * 64 * 8 = 48 KB
    hipLaunchKernelGGL(sample_verify_kernel, dim3(v.batch), dim3(256), lds, s, v);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// losses of SAR-SFT (Methods, "Semi-Autoregressive Finetuning"): -log softmax(row)[label] per row
// ------------------------------------------------------------------------------------------
// Both L_AR and L_SAR are sums of such terms; which rows and labels enter is the caller's (the
// dataloader's) business.  One workgroup per row: maximum, sum of exponentials (each thread over its
// strided elements, then a fixed tree: the result does not depend on timing), then the term.  A
// second launch adds the rows up in row order in one thread.

__global__ __launch_bounds__(1024) void nll_rows_kernel(const float* __restrict__ logits, const int32_t* __restrict__ labels,
                                                        int vocab, float* __restrict__ row_loss, int32_t* faults) {
    __shared__ float sh[16];
    const int row = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int label = labels[row];
    if (label < 0 || label >= vocab) {  // ignored row (negative) or a label outside the vocabulary (counted)
        if (tid == 0) {
            row_loss[row] = 0.f;
            if (label >= vocab) atomicAdd(faults, 1);
        }
        return;
    }
    const float* __restrict__ x = logits + (size_t)row * vocab;
    float mx = -INFINITY;
    for (int i = tid; i < vocab; i += 1024) mx = fmaxf(mx, x[i]);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
    if (lane == 0) sh[wave] = mx;
    __syncthreads();
    mx = sh[0];
    for (int w = 1; w < 16; ++w) mx = fmaxf(mx, sh[w]);
    __syncthreads();
    float sum = 0.f;
    for (int i = tid; i < vocab; i += 1024) sum += expf(x[i] - mx);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o, 64);
    if (lane == 0) sh[wave] = sum;
    __syncthreads();
    if (tid == 0) {
        float tot = 0.f;
        for (int w = 0; w < 16; ++w) tot += sh[w];
        row_loss[row] = -(x[label] - mx - logf(tot));
    }
}

__global__ void nll_sum_kernel(const float* row_loss, const int32_t* labels, int rows, int vocab, float* loss_sum,
                               int32_t* n_terms) {
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    float tot = 0.f;
    int n = 0;
    for (int r = 0; r < rows; ++r) {
        const int label = labels[r];
        if (label >= 0 && label < vocab) {
            tot += row_loss[r];
            ++n;
        }
    }
    *loss_sum = tot;
    if (n_terms) *n_terms = n;
}

hipError_t launch_nll(const float* logits, const int32_t* labels, int rows, int vocab, float* row_loss, float* loss_sum,
                      int32_t* n_terms, int32_t* faults, hipStream_t s) {
    if (rows < 1 || vocab < 1) return hipErrorInvalidValue;
    hipLaunchKernelGGL(nll_rows_kernel, dim3(rows), dim3(1024), 0, s, logits, labels, vocab, row_loss, faults);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(nll_sum_kernel, dim3(1), dim3(64), 0, s, row_loss, labels, rows, vocab, loss_sum, n_terms);
    return hipGetLastError();
}

// commit: len += clamp(accepted, 0, hi) + 1; rollback: len = max(0, len - n)
__global__ void kv_len_kernel(int32_t* len, int batch, const int32_t* delta_dev, int delta_all, int sign, int clamp_hi,
                              int capacity) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= batch) return;
    int d = delta_dev ? delta_dev[b] : delta_all;
    if (sign > 0) d = min(max(d, 0), clamp_hi) + 1; else d = max(d, 0);
    len[b] = min(max(len[b] + sign * d, 0), capacity);
}

hipError_t launch_kv_len_update(int32_t* len, int batch, const int32_t* delta_dev, int delta_all, int sign,
                                int clamp_hi, int capacity, hipStream_t s) {
    hipLaunchKernelGGL(kv_len_kernel, dim3(ceil_div(batch, 64)), dim3(64), 0, s, len, batch, delta_dev, delta_all,
                       sign, clamp_hi, capacity);
    return hipGetLastError();
}

}  // namespace space
