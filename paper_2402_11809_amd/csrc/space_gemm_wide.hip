// Projection kernel for many rows (prompt chunks, batches of blocks): out[m, n] = sum_k x[m, k] * W[n, k]
// for m of a few hundred and more.  The paper's premise (decoding is bound by the weight stream, so
// the extra rows of the block are free) ends where the matrix unit becomes the limit: with two
// products per element (hi and lo activation plane) that is at roughly 190 rows on this chip.  Here
// the arithmetic has to be fed, not the weight stream:
//   * a workgroup of 8 waves owns 16 weight tiles x up to 8 row tiles (256 x 128 outputs); its waves
//     split the weight rows, so each wave streams its own 2 packed weight tiles per contraction tile
//     straight into MFMA operand registers (buffer loads, no LDS, the same packed matrix the skinny
//     kernel reads; a ring of 2 tiles per weight tile row is in flight);
//   * the activation planes of the row tiles go from global memory straight into LDS (buffer loads that
//     write LDS; double buffered, 2 contraction tiles per barrier) and are read from there by all
//     waves, two row tiles at a time, one such group ahead of the MFMAs that use it;
//   * each wave owns complete sums of its tiles, so the epilogues (fp32 partials, SwiGLU, argmax) run
//     out of registers with no reduction across waves, except the argmax, which merges the waves
//     through LDS;
//   * a CU gets through one such workgroup per unit of time however many it holds (two fit: 119
//     registers, 64 KB of LDS), so what a launch costs is the work of its busiest CU.  The rows of a
//     weight group are therefore cut into pieces of 8, 6, 4 or 2 row tiles (WideParts, chosen by the
//     host: by default pieces of 8 and one for the rest, else what space_tune_rows measured);
//   * the pieces of one weight group get workgroup indices that differ by 8 (same XCD, about the same
//     time), so the weights cross HBM once and the siblings hit L2.
// Per contraction tile a full workgroup moves 16 KB of weights and 16 KB of activation planes for
// 32 MFMAs per wave.
#include "space_device.h"
#include "space_kernels.h"

#include <limits.h>
#include <math.h>
#include <stdlib.h>
#include <type_traits>

namespace space {

namespace {

// Measured at 7B shapes (waves x weight tiles per wave): 8 x 2 with two workgroups per CU beat 8 x 4
// and 4 x 8 with one per CU; a split of the 8 waves into 4 weight quarters x 2 row halves (half the LDS
// reads per MFMA, every weight tile requested by two waves) was 1-4 % slower; deeper rings spilled or
// changed nothing.
constexpr int kWideStage = 2;   // contraction tiles per LDS stage
constexpr int kWideWaves = 8;   // waves per workgroup
constexpr int kWideTiles = 2;   // weight tiles per wave: a workgroup covers 256 weight rows
constexpr int kWideDepth = 2;   // weight tiles in flight per wave and tile row

template <int W, int R, int KS, int DA, int EPI>
__global__ __launch_bounds__(64 * W, 2 * W / 4) void gemm_wide_kernel(GemmLaunch g, int ksplit, int n_groups, int kt_per_split,
                                                                       WideParts parts) {
    constexpr int T = kWideRowTiles, TB = 2, GMAX = T / TB;
    static_assert(R % 2 == 0 && W == 8 && DA == KS && T == 8, "tile counts");
#if defined(__HIP_DEVICE_COMPILE__)  // the host pass only needs the launch stub: the body is device code throughout (LDS address casts, inline assembly)
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // Which piece.  Two launch orders (parts.by_size): weight group by weight group, 8 groups (x
    // contraction splits) at a time with all their pieces, the large ones first (0); or size class by
    // size class over all weight groups, i.e. every large piece of the launch before any smaller one
    // (1: better once the launch no longer fits the chip at once, the small pieces then fill the gaps at
    // the end).  Either way the pieces of one weight group sit 8 indices apart (same XCD, for order 0
    // also about the same time, so that its weights cross HBM once and the siblings hit L2).
    const int n_gk = n_groups * ksplit, gk8 = (n_gk + 7) / 8 * 8;
    const int n_pieces = parts.count[0] + parts.count[1] + parts.count[2] + parts.count[3];
    int G = 0, row_tile0 = 0, gi;
    if (parts.by_size) {
        int idx = blockIdx.x, cnt = 1;
#pragma unroll
        for (int c = 0; c < GMAX; ++c) {
            if (G == 0) {
                const int size = gk8 * parts.count[c];
                if (idx < size) {
                    G = GMAX - c;
                    cnt = parts.count[c];
                } else {
                    idx -= size;
                    row_tile0 += parts.count[c] * TB * (GMAX - c);
                }
            }
        }
        if (G == 0) return;  // whole workgroup, before any barrier
        const int q = idx >> 3;
        gi = (q / cnt) * 8 + (idx & 7);
        row_tile0 += (q % cnt) * TB * G;
    } else {
        const int q = blockIdx.x >> 3;
        gi = (q / n_pieces) * 8 + (blockIdx.x & 7);
        int piece = q % n_pieces;
#pragma unroll
        for (int c = 0; c < GMAX; ++c) {
            if (G == 0) {
                if (piece < parts.count[c]) {
                    G = GMAX - c;
                    row_tile0 += piece * TB * G;
                } else {
                    piece -= parts.count[c];
                    row_tile0 += parts.count[c] * TB * (GMAX - c);
                }
            }
        }
    }
    if (gi >= n_gk) return;
    const int bx = gi % n_groups, s = gi / n_groups;
    const int m_rows = min(g.m - row_tile0 * 16, 16 * TB * G);
    if (m_rows <= 0) return;
    const int t_run = (m_rows + 15) >> 4;
    // Contraction range of this split: a multiple of DA tiles (the host rounds; tiles past k_tiles exist
    // in the packed matrix as zeros, and the activation buffers are finite there).
    const int k0 = s * kt_per_split, k1 = min(k0 + kt_per_split, (g.w.k_tiles + DA - 1) / DA * DA);

    // weights: tile (nt, kt) of the packed matrix sits at tile index ck(kt) + cr(nt)
    const int nt0 = (bx * W + wave) * R;
    const int nt_last = g.w.groups * g.w.r_pack - 1;  // padded tile grid
    // buffer loads: resource of the whole packed matrix (under 4 GB, the host checks) + the tile's byte
    // offset in a scalar register + the lane's 16 bytes: no 64-bit address arithmetic per load
    const __amdgpu_buffer_rsrc_t wrs = __builtin_amdgcn_make_buffer_rsrc((void*)g.w.data, 0, -1, 0x00020000);
    const int lane16 = lane * 16;
    auto ldw = [&](uint32_t unit) -> u32x4 { return __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(wrs, lane16, (int)(unit * 16u), 0)); };
    uint32_t cr[R];  // in 16-byte units
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int nt = min(nt0 + r, nt_last);
        cr[r] = __builtin_amdgcn_readfirstlane((uint32_t)((nt / g.w.r_pack) * 4 * g.w.r_pack + nt % g.w.r_pack) * 64u);
    }
    const uint32_t sg4 = (uint32_t)g.w.splits * g.w.groups * 4;
    auto ck = [&](int kt) -> uint32_t {  // wave uniform, kept in scalar registers
        const int rq = kt / g.w.lq, i = kt - rq * g.w.lq;
        return __builtin_amdgcn_readfirstlane(((uint32_t)i * sg4 + (uint32_t)(rq >> 2) * g.w.groups * 4 + (rq & 3)) * g.w.r_pack * 64u);
    };

    // activations: the planes of this piece's row tiles at contraction tile kt start at unit (16 bytes)
    // kt * xkt + row_tile0 * 128.  The LDS copy always has the full-tile format (unit t*128 + plane*64
    // + l for lane l), so the compact last row tile of the matrix is spread out while it is copied;
    // rows and columns that do not exist get a copy of an existing unit (finite, and a token only ever
    // meets its own column; the epilogues drop them).
    // Thread i copies unit w = i % 128 of the row tiles i/128 and i/128 + 4 (those the piece has): as
    // buffer loads that write LDS directly (no registers, no LDS write instructions); the 64 lanes of a
    // wave land at the wave's LDS base + 16 l, their sources are per lane.
    constexpr int NS = T * 2 / W;
    const u32x4* xp = (const u32x4*)g.x + (size_t)row_tile0 * 128;
    const size_t xkt = (size_t)(g.xs.row_tiles - 1) * 128 + 8 * g.xs.last_cols;
    const int lc = g.xs.last_cols;
    const int w_full = threadIdx.x & 127, tile_w = wave >> 1;
    const int w_rag = (w_full >> 4) * lc + min(w_full & 15, lc - 1);
    const int rag_tile = g.xs.row_tiles - 1 - row_tile0;  // index in this piece of the compact tile (may be >= t_run)
    int voff[NS];  // byte offset of this lane's source inside a contraction tile
#pragma unroll
    for (int i = 0; i < NS; ++i) {
        const int t = min(tile_w + (W / 2) * i, t_run - 1);
        voff[i] = (t * 128 + (t == rag_tile ? w_rag : w_full)) * 16;
    }
    const int wave_unit = tile_w * 128 + (wave & 1) * 64;  // first LDS unit of this wave's copies (+ 64 W i)
    __shared__ u32x4 lds[2][KS][T * 128];
    const __amdgpu_buffer_rsrc_t xrs = __builtin_amdgcn_make_buffer_rsrc((void*)xp, 0, 0x7fffffff, 0x00020000);
    // The LDS reads are written by hand: the compiler makes every LDS read it knows of wait for all
    // outstanding copies into LDS, i.e. for the stage that was just requested.  4 reads (hi and lo
    // plane of two row tiles) per group; the wait names how many younger reads may stay outstanding and
    // carries the registers, so that no MFMA can move above it.
    const unsigned lds_lane = (unsigned)(size_t)(__attribute__((address_space(3))) char*)&lds[0][0][0] + lane * 16;
    auto rd = [&](u32x4(&bb)[2 * TB], unsigned addr) {
        asm volatile(
            "ds_read_b128 %0, %4\n\tds_read_b128 %1, %4 offset:1024\n\tds_read_b128 %2, %4 offset:2048\n\tds_read_b128 %3, %4 offset:3072"
            : "=&v"(bb[0]), "=&v"(bb[1]), "=&v"(bb[2]), "=&v"(bb[3])
            : "v"(addr));
    };
    auto wait_for = [&](u32x4(&bb)[2 * TB], bool younger) {  // younger: the next group's reads are in flight
        if (younger) asm volatile("s_waitcnt lgkmcnt(4)" : "+v"(bb[0]), "+v"(bb[1]), "+v"(bb[2]), "+v"(bb[3]));
        else asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(bb[0]), "+v"(bb[1]), "+v"(bb[2]), "+v"(bb[3]));
    };

    // the argmax epilogue merges the waves through these (one copy, whatever the piece size)
    __shared__ float s_val[EPI == EPI_ARGMAX ? W : 1][EPI == EPI_ARGMAX ? T * 16 : 1];
    __shared__ int s_idx[EPI == EPI_ARGMAX ? W : 1][EPI == EPI_ARGMAX ? T * 16 : 1];
    // The loop over the contraction for a piece of GC groups of two row tiles: nothing in it is
    // conditional, the LDS reads of a group are issued one group ahead of the MFMAs that use them.  A
    // last row tile that the matrix does not have is computed on copies of existing rows and dropped.
    auto run = [&](auto gc_tag) {
        constexpr int GC = decltype(gc_tag)::value, TG = TB * GC;  // row tiles of this piece
        // copies of a stage: of its NS row tiles a wave copies those the piece has (decided at compile
        // time where the piece size settles it)
        auto copy_stage = [&](int to, int kt_first) {
#pragma unroll
            for (int j = 0; j < KS; ++j) {
                const int kt = min(kt_first + j, k1 - 1);
#pragma unroll
                for (int i = 0; i < NS; ++i) {
                    constexpr int kHalf = W / 2;
                    if (kHalf * i >= TG) continue;
                    if (kHalf * (i + 1) <= TG || tile_w + kHalf * i < TG)  // wave uniform
                        __builtin_amdgcn_raw_ptr_buffer_load_lds(xrs, (__attribute__((address_space(3))) void*)&lds[to][j][wave_unit + 64 * W * i],
                                                                 16, voff[i], (int)(kt * xkt * 16), 0, 0);
                }
            }
        };
        f32x4 acc[R][TG];
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int t = 0; t < TG; ++t) acc[r][t] = f32x4{0.f, 0.f, 0.f, 0.f};
        auto mfma_group = [&](const u32x4(&aj)[R], const u32x4(&bc)[2 * TB], int tb) {
            // hi planes of all R * TB tiles first, then the lo planes: R * TB MFMAs lie between the two that
            // add into the same accumulator
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int t = 0; t < TB; ++t) acc[r][tb + t] = mfma16(aj[r], bc[2 * t], acc[r][tb + t]);
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int t = 0; t < TB; ++t) acc[r][tb + t] = mfma16(aj[r], bc[2 * t + 1], acc[r][tb + t]);
        };

        // prologue: first stage of activations on its way to LDS, first DA weight tiles in flight.  Every
        // load of the loop is unconditional (indices clamped to the range) so that the waits can be counted.
        u32x4 a[DA][R];
        copy_stage(0, k0);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < DA; ++j) {
            const uint32_t c = ck(min(k0 + j, k1 - 1));
#pragma unroll
            for (int r = 0; r < R; ++r) a[j][r] = ldw(c + cr[r]);
        }
        __builtin_amdgcn_sched_barrier(0);
        // the copies are complete when at most the DA * R weight loads issued behind them are outstanding
        __builtin_amdgcn_s_waitcnt(0x0070 | (DA * R));
        __builtin_amdgcn_s_barrier();

        int buf = 0;
        for (int kt0 = k0; kt0 < k1; kt0 += DA) {
            copy_stage(buf ^ 1, kt0 + KS);  // the other buffer: everybody's reads of it ended before the last barrier
            __builtin_amdgcn_sched_barrier(0);
            const unsigned rbase = lds_lane + buf * (unsigned)(KS * T * 128 * 16);
            u32x4 b[2][2 * TB];
            rd(b[0], rbase);
#pragma unroll
            for (int j = 0; j < KS; ++j) {
                const uint32_t cn = ck(min(kt0 + j + DA, k1 - 1));
#pragma unroll
                for (int gi2 = 0; gi2 < GC; ++gi2) {
                    const int gq = j * GC + gi2;  // group index in the stage
                    u32x4(&bc)[2 * TB] = b[gq & 1];
                    if (gq + 1 < KS * GC) rd(b[(gq + 1) & 1], rbase + (unsigned)(((gq + 1) / GC) * T * 128 * 16 + ((gq + 1) % GC) * TB * 128 * 16));
                    wait_for(bc, gq + 1 < KS * GC);
                    mfma_group(a[j], bc, gi2 * TB);
                    __builtin_amdgcn_sched_barrier(0);
                }
                // the tiles are consumed: their successors DA contraction tiles ahead take the registers
#pragma unroll
                for (int r = 0; r < R; ++r) a[j][r] = ldw(cn + cr[r]);
                __builtin_amdgcn_sched_barrier(0);
            }
            // own copies landed (only the KS * R weight loads issued behind them may be outstanding) and own
            // reads of this buffer done; then everybody's
            __builtin_amdgcn_s_waitcnt(0x0070 | (KS * R));
            __builtin_amdgcn_s_barrier();
            buf ^= 1;
        }
    

        // ---- epilogue out of registers: lane l holds, of tile (r, t), token 16 t + l%16 and the 4
        // weight rows 16 nt + 4 (l/16) .. + 3
        const int N = g.w.n;
        const int tok_l = lane & 15, n_l = 4 * (lane >> 4);
        if (EPI == EPI_F32 || EPI == EPI_ARGMAX) {
            float* outp = g.out ? g.out + (size_t)s * g.split_stride + (size_t)row_tile0 * 16 * g.ldo : nullptr;
            if (outp) {
                const bool vec_ok = (g.ldo & 3) == 0;
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    const int nt = nt0 + r;
                    if (nt >= g.w.n_tiles) break;
                    const int n = nt * 16 + n_l;
#pragma unroll
                    for (int t = 0; t < TG; ++t) {
                        const int tok = 16 * t + tok_l;
                        if (tok >= m_rows) continue;
                        float* o = outp + (size_t)tok * g.ldo + n;
                        if (vec_ok && n + 3 < N) {
                            *(f32x4*)o = acc[r][t];
                        } else {
#pragma unroll
                            for (int e = 0; e < 4; ++e)
                                if (n + e < N) o[e] = acc[r][t][e];
                        }
                    }
                }
            }
        }
        if (EPI == EPI_ARGMAX) {
            // per token the (max, lowest index) pair over this workgroup's columns: lane, then the 4 lane
            // groups of a token, then the waves along the weight rows in order
#pragma unroll
            for (int t = 0; t < TG; ++t) {
                float best = -INFINITY;
                int bidx = INT_MAX;
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    const int nt = nt0 + r;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int n = nt * 16 + n_l + e;
                        const float v = acc[r][t][e];
                        if (nt < g.w.n_tiles && n < N && v > best) { best = v; bidx = n; }
                    }
                }
#pragma unroll
                for (int off = 16; off <= 32; off <<= 1) {
                    const float ov = __shfl_xor(best, off, 64);
                    const int oi = __shfl_xor(bidx, off, 64);
                    if (ov > best || (ov == best && oi < bidx)) { best = ov; bidx = oi; }
                }
                if (lane < 16) {
                    s_val[wave][16 * t + lane] = best;
                    s_idx[wave][16 * t + lane] = bidx;
                }
            }
            __syncthreads();
            const int tok = threadIdx.x;
            if (tok < T * 16 && tok < m_rows) {
                float best = s_val[0][tok];
                int bidx = s_idx[0][tok];
                for (int w = 1; w < W; ++w) {
                    const float ov = s_val[w][tok];
                    const int oi = s_idx[w][tok];
                    if (ov > best || (ov == best && oi < bidx)) { best = ov; bidx = oi; }
                }
                g.arg_val[(size_t)(row_tile0 * 16 + tok) * g.arg_groups + bx] = best;
                g.arg_idx[(size_t)(row_tile0 * 16 + tok) * g.arg_groups + bx] = bidx;
            }
        }
        if (EPI == EPI_SWIGLU) {  // even tiles are gate rows, odd tiles the matching up rows
#pragma unroll
            for (int p = 0; p < R / 2; ++p) {
                const int j = (((nt0 >> 1) + p) * 16) + n_l;
                if (j >= g.ffn) break;
#pragma unroll
                for (int t = 0; t < TG; ++t) {
                    const int tok = 16 * t + tok_l;
                    if (tok >= m_rows) continue;
                    const int m = row_tile0 * 16 + tok;
                    uint32_t hi[4], lo[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        // silu(g) * u with the hardware exp2 / reciprocal (about 1 ulp each)
                        const float gg = acc[2 * p][t][e];
                        const float v = gg * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * gg)) *
                                        acc[2 * p + 1][t][e];
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
    };
    switch (G) {
        case 4: run(std::integral_constant<int, 4>{}); break;
        case 3: run(std::integral_constant<int, 3>{}); break;
        case 2: run(std::integral_constant<int, 2>{}); break;
        default: run(std::integral_constant<int, 1>{}); break;
    }

#endif
}

template <int W, int R, int EPI>
hipError_t launch_wide_r(const GemmLaunch& g, int ksplit, int n_groups, int kt_per_split, const WideParts& parts, hipStream_t s) {
    int pieces = 0;
    for (int c = 0; c < 4; ++c) pieces += parts.count[c];
    const dim3 grid(8 * ceil_div(n_groups * ksplit, 8) * pieces), block(64 * W);
    hipLaunchKernelGGL((gemm_wide_kernel<W, R, kWideStage, kWideDepth, EPI>), grid, block, 0, s, g, ksplit, n_groups, kt_per_split, parts);
    return hipGetLastError();
}

}  // namespace

WidePlan plan_gemm_wide(const PackedW& w, int m, GemmEpilogue epi, int max_splits, int force_ksplit) {
    WidePlan p{};
    const int row_tiles = ceil_div(m, 16), groups = ceil_div(row_tiles, 2);
    p.tiles_per_wave = kWideTiles;
    p.n_groups = ceil_div(w.n_tiles, kWideWaves * kWideTiles);
    // rows: pieces of 8 row tiles and one for the rest, the large ones first over the whole launch
    p.parts.count[0] = groups / 4;
    if (groups % 4) p.parts.count[4 - groups % 4] = 1;
    p.parts.by_size = 1;
    int pieces = 0;
    for (int c = 0; c < 4; ++c) pieces += p.parts.count[c];
    // Split of the contraction (plain sums only): a CU works through its share of the workgroups at a
    // rate that hardly depends on how many it holds at once, so the time goes with
    // ceil(workgroups / CUs) * contraction tiles per workgroup; every doubling costs a little for the
    // partial sums, and a split keeps at least 16 tiles.
    const int smax = (epi == EPI_F32) ? (max_splits < 4 ? max_splits : 4) : 1;
    double best = 1e30;
    p.ksplit = 1;
    for (int ks = 1; ks <= smax; ks *= 2) {
        if (ks > 1 && w.k_tiles / ks < 16) break;
        const double cost = (double)ceil_div(p.n_groups * pieces * ks, 256) * ceil_div(w.k_tiles, ks) * (ks == 1 ? 1.0 : ks == 2 ? 1.04 : 1.08);
        if (cost < best) { best = cost; p.ksplit = ks; }
    }
    if (force_ksplit > 0 && epi == EPI_F32) p.ksplit = force_ksplit < smax ? force_ksplit : smax;
    p.kt_per_split = round_up(ceil_div(w.k_tiles, p.ksplit), kWideDepth);
    p.ksplit = ceil_div(w.k_tiles, p.kt_per_split);  // no empty split
    return p;
}

hipError_t launch_gemm_wide(const GemmLaunch& g0, const WidePlan& p, GemmEpilogue epi, hipStream_t s) {
    GemmLaunch g = g0;
    int groups = 0;
    for (int c = 0; c < 4; ++c) {
        if (p.parts.count[c] < 0 || (p.parts.by_size != 0 && p.parts.by_size != 1)) return hipErrorInvalidValue;
        groups += p.parts.count[c] * (4 - c);
    }
    if (g.m < 1 || groups != ceil_div(ceil_div(g.m, 16), 2) || g.row_tile0 != 0 || g.w.k_tiles < 1 ||
        g.xs.row_tiles != ceil_div(g.m, 16) || g.xs.last_cols != g.m - 16 * (g.xs.row_tiles - 1))
        return hipErrorInvalidValue;
    if (p.ksplit < 1 || p.kt_per_split < 1 || p.kt_per_split % kWideDepth || (p.ksplit - 1) * p.kt_per_split >= g.w.k_tiles ||
        p.ksplit * p.kt_per_split < g.w.k_tiles || round_up(g.w.k_tiles, kWideDepth) > g.w.k_tiles_pad() ||
        p.n_groups != ceil_div(g.w.n_tiles, kWideWaves * p.tiles_per_wave))
        return hipErrorInvalidValue;
    if (epi != EPI_F32 && p.ksplit != 1) return hipErrorInvalidValue;
    if (g.w.bytes() >= ((size_t)1 << 32)) return hipErrorInvalidValue;  // the kernel addresses the matrix with 32-bit byte offsets
    if (epi == EPI_ARGMAX && p.n_groups > g.arg_groups) return hipErrorInvalidValue;
    if (p.tiles_per_wave != kWideTiles) return hipErrorInvalidValue;
    switch (epi) {
        case EPI_F32: return launch_wide_r<kWideWaves, kWideTiles, EPI_F32>(g, p.ksplit, p.n_groups, p.kt_per_split, p.parts, s);
        case EPI_SWIGLU: return launch_wide_r<kWideWaves, kWideTiles, EPI_SWIGLU>(g, p.ksplit, p.n_groups, p.kt_per_split, p.parts, s);
        case EPI_ARGMAX: return launch_wide_r<kWideWaves, kWideTiles, EPI_ARGMAX>(g, p.ksplit, p.n_groups, p.kt_per_split, p.parts, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace space
