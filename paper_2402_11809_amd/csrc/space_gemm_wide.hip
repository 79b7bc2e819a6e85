// Projection kernel for many rows (prompt chunks, batches of blocks): out[m, n] = sum_k x[m, k] * W[n, k]
// for m of a few hundred and more.  The paper's premise (decoding is bound by the weight stream, so
// the extra rows of the block are free) ends where the matrix unit becomes the limit: with two
// products per element (hi and lo activation plane) that is at roughly 190 rows on this chip.  Here
// the arithmetic has to be fed, not the weight stream:
//   * a workgroup of W waves owns W*R weight tiles x T row tiles (256 x 128 outputs for W = 8, R = 2,
//     T = 8); its waves split the weight rows, so each wave streams its own R packed weight tiles per
//     contraction tile straight into MFMA operand registers (no LDS, same packed matrix the skinny
//     kernel reads; a ring of DA tiles per weight tile row is in flight);
//   * the activation planes of the T row tiles are copied once per workgroup into LDS (double
//     buffered, KS contraction tiles per barrier) and read from there by all waves, TB row tiles at
//     a time;
//   * each wave owns complete sums of its R*T tiles, so the epilogues (fp32 partials, SwiGLU, argmax)
//     run out of registers with no reduction across waves, except the argmax, which merges the waves through LDS;
//   * row passes of one weight group get workgroup indices that differ by 8 (same XCD, about the
//     same time), so the weights cross HBM once and the sibling passes hit L2;
//   * 124 registers and 64 KB of LDS: two workgroups per CU, one runs while the other waits.
// Per contraction tile a workgroup moves 16 KB of weights and 16 KB of activation planes for
// 2*R*T = 32 MFMAs per wave.  What bounds it is what one CU can pull from L2 (about 45 GB/s here,
// whatever is in flight): two such workgroups would need 75 GB/s to keep the matrix unit busy.
#include "space_device.h"
#include "space_kernels.h"

#include <limits.h>
#include <math.h>
#include <stdlib.h>

namespace space {

namespace {

// Measured at 7B shapes (waves x weight tiles per wave): 8 x 2 with two workgroups per CU beat 8 x 4
// and 4 x 8 with one per CU (the same work per unit of time inside a full round, but whole 512 x 128
// workgroups leave more CUs idle in the last round); deeper rings spilled or changed nothing.
constexpr int kWideStage = 2;   // contraction tiles per LDS stage
constexpr int kWideWaves = 8;   // waves per workgroup
// Waves along the rows (WT): 1 = every wave owns its 2 weight tiles for all 128 rows; 2 = 4 weight tiles
// for 64 rows each (half the LDS reads per MFMA, every weight tile requested by two waves): measured 1-4 %
// slower at 512-1024 rows, so the LDS reads are not what holds the kernel back.
constexpr int kWideRowSplit = 1;
constexpr int kWideTiles = 2 * kWideRowSplit;   // weight tiles per wave: a workgroup covers 256 weight rows x 128 rows
constexpr int kWideDepth = 2;                   // weight tiles in flight per wave and tile row
constexpr int kWideTB = 2 / kWideRowSplit;      // row tiles whose operands are read from LDS at a time

template <int W, int WT, int R, int T, int KS, int DA, int TB, int EPI>
__global__ __launch_bounds__(64 * W, 2 * W / 4) void gemm_wide_kernel(GemmLaunch g, int ksplit, int n_groups, int kt_per_split) {
    static_assert(R % 2 == 0 && (T * 2) % W == 0 && (W == 4 || W == 8) && DA % KS == 0 && (WT == 1 || WT == 2) && T % WT == 0 &&
                      (T / WT) % TB == 0 && (TB == 1 || TB == 2),
                  "tile counts");
#if defined(__HIP_DEVICE_COMPILE__)  // the host pass only needs the launch stub: the body is device code throughout (LDS address casts, inline assembly)
    constexpr int NS = T * 2 / W;  // 16-byte units a thread copies per contraction tile
    constexpr int WN = W / WT;     // waves along the weight rows
    constexpr int TW = T / WT;     // row tiles per wave
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wave_n = wave / WT, t_off = (wave % WT) * TW;  // this wave's weight tiles and first row tile
    const int q = blockIdx.x >> 3;
    const int pass = q % g.passes;
    const int gi = (q / g.passes) * 8 + (blockIdx.x & 7);
    if (gi >= n_groups * ksplit) return;  // whole workgroup, before any barrier
    const int bx = gi % n_groups, s = gi / n_groups;
    const int row_tile0 = pass * T;
    const int m_rows = min(g.m - pass * 16 * T, 16 * T);
    const int t_run = (m_rows + 15) >> 4;
    // Contraction range of this split: a multiple of DA tiles (the host rounds; tiles past k_tiles exist
    // in the packed matrix as zeros, and the activation buffers are finite there).
    const int k0 = s * kt_per_split, k1 = min(k0 + kt_per_split, (g.w.k_tiles + DA - 1) / DA * DA);

    // weights: tile (nt, kt) of the packed matrix sits at tile index ck(kt) + cr(nt)
    const int nt0 = (bx * WN + wave_n) * R;
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

    // activations: the planes of this pass's row tiles at contraction tile kt start at unit (16 bytes)
    // kt * xkt + row_tile0 * 128.  The LDS copy always has the full-tile format (unit t*128 + plane*64
    // + l for lane l), so the compact last row tile of the matrix is spread out while it is copied;
    // rows and columns that do not exist get a copy of an existing unit (finite, and a token only ever
    // meets its own column; the epilogues drop them).
    // Thread i copies unit w = i % 128 of the row tiles i/128, i/128 + W/2, ...: as buffer loads that
    // write LDS directly (no registers, no LDS write instructions); the 64 lanes of a wave land at the
    // wave's LDS base + 16 l, their sources are per lane.
    const u32x4* xp = (const u32x4*)g.x + (size_t)row_tile0 * 128;
    const size_t xkt = (size_t)(g.xs.row_tiles - 1) * 128 + 8 * g.xs.last_cols;
    const int lc = g.xs.last_cols;
    const int w_full = threadIdx.x & 127, tile_w = threadIdx.x >> 7;
    const int w_rag = (w_full >> 4) * lc + min(w_full & 15, lc - 1);
    const int rag_tile = g.xs.row_tiles - 1 - row_tile0;  // index in this pass of the compact tile (may be >= t_run)
    int voff[NS];  // byte offset of this lane's source inside a contraction tile
#pragma unroll
    for (int i = 0; i < NS; ++i) {
        const int t = min(tile_w + (W / 2) * i, t_run - 1);
        voff[i] = (t * 128 + (t == rag_tile ? w_rag : w_full)) * 16;
    }
    const int wave_unit = (wave >> 1) * 128 + (wave & 1) * 64;  // first LDS unit of this wave's copies (+ 64 W i)

    __shared__ u32x4 lds[2][KS][T * 128];
    const __amdgpu_buffer_rsrc_t xrs = __builtin_amdgcn_make_buffer_rsrc((void*)xp, 0, 0x7fffffff, 0x00020000);
    auto copy_stage = [&](int to, int kt_first) {
#pragma unroll
        for (int j = 0; j < KS; ++j) {
            const int kt = min(kt_first + j, k1 - 1);
#pragma unroll
            for (int i = 0; i < NS; ++i)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(xrs, (__attribute__((address_space(3))) void*)&lds[to][j][wave_unit + 64 * W * i], 16,
                                                         voff[i], (int)(kt * xkt * 16), 0, 0);
        }
    };
    // The LDS reads are written by hand: the compiler makes every LDS read it knows of wait for all
    // outstanding copies into LDS, i.e. for the stage that was just requested.  2 TB reads (hi and lo
    // plane of TB row tiles) per group; the wait names how many younger reads may stay outstanding and
    // carries the registers, so that no MFMA can move above it.
    const unsigned lds_lane = (unsigned)(size_t)(__attribute__((address_space(3))) char*)&lds[0][0][0] + (t_off * 128 + lane) * 16;
    auto rd = [&](u32x4(&bb)[2 * TB], unsigned addr) {
        if constexpr (TB == 2)
            asm volatile(
                "ds_read_b128 %0, %4\n\tds_read_b128 %1, %4 offset:1024\n\tds_read_b128 %2, %4 offset:2048\n\tds_read_b128 %3, %4 offset:3072"
                : "=&v"(bb[0]), "=&v"(bb[1]), "=&v"(bb[2]), "=&v"(bb[3])
                : "v"(addr));
        else
            asm volatile("ds_read_b128 %0, %2\n\tds_read_b128 %1, %2 offset:1024" : "=&v"(bb[0]), "=&v"(bb[1]) : "v"(addr));
    };
    auto wait_for = [&](u32x4(&bb)[2 * TB], bool younger) {  // younger: the next group's reads are in flight
        if constexpr (TB == 2) {
            if (younger) asm volatile("s_waitcnt lgkmcnt(4)" : "+v"(bb[0]), "+v"(bb[1]), "+v"(bb[2]), "+v"(bb[3]));
            else asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(bb[0]), "+v"(bb[1]), "+v"(bb[2]), "+v"(bb[3]));
        } else {
            if (younger) asm volatile("s_waitcnt lgkmcnt(2)" : "+v"(bb[0]), "+v"(bb[1]));
            else asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(bb[0]), "+v"(bb[1]));
        }
    };

    f32x4 acc[R][TW];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int t = 0; t < TW; ++t) acc[r][t] = f32x4{0.f, 0.f, 0.f, 0.f};
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

    static_assert(DA == KS, "one LDS stage per ring of weight tiles");
    constexpr int G = TW / TB;  // groups of row tiles per contraction tile and wave
    // A pass is "full" when it has all T row tiles: then nothing in the loop is conditional and the LDS
    // reads of a group are issued one group ahead of the MFMAs that use them.  The short last pass of a
    // ragged row count skips the groups it does not have and reads each group right before its MFMAs
    // (within a group, missing tiles are computed on copies of existing rows and dropped in the epilogue).
    const bool full = t_run == T;

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

    // own copies landed (only the KS * R weight loads issued behind them may be outstanding) and own reads
    // of this buffer done; then everybody's
    auto end_stage = [&]() {
        __builtin_amdgcn_s_waitcnt(0x0070 | (KS * R));
        __builtin_amdgcn_s_barrier();
    };
    if (full) {
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
                for (int gi2 = 0; gi2 < G; ++gi2) {
                    const int gq = j * G + gi2;  // group index in the stage
                    u32x4(&bc)[2 * TB] = b[gq & 1];
                    if (gq + 1 < KS * G) rd(b[(gq + 1) & 1], rbase + (unsigned)(((gq + 1) / G) * T * 128 * 16 + ((gq + 1) % G) * TB * 128 * 16));
                    wait_for(bc, gq + 1 < KS * G);
                    mfma_group(a[j], bc, gi2 * TB);
                    __builtin_amdgcn_sched_barrier(0);
                }
                // the tiles are consumed: their successors DA contraction tiles ahead take the registers
#pragma unroll
                for (int r = 0; r < R; ++r) a[j][r] = ldw(cn + cr[r]);
                __builtin_amdgcn_sched_barrier(0);
            }
            end_stage();
            buf ^= 1;
        }
    } else {
        int buf = 0;
        for (int kt0 = k0; kt0 < k1; kt0 += DA) {
            copy_stage(buf ^ 1, kt0 + KS);
            __builtin_amdgcn_sched_barrier(0);
            const unsigned rbase = lds_lane + buf * (unsigned)(KS * T * 128 * 16);
#pragma unroll
            for (int j = 0; j < KS; ++j) {
                const uint32_t cn = ck(min(kt0 + j + DA, k1 - 1));
#pragma unroll
                for (int gi2 = 0; gi2 < G; ++gi2) {
                    if (t_off + gi2 * TB < t_run) {  // wave uniform
                        u32x4 bc[2 * TB];
                        rd(bc, rbase + (unsigned)(j * T * 128 * 16 + gi2 * TB * 128 * 16));
                        wait_for(bc, false);
                        mfma_group(a[j], bc, gi2 * TB);
                    }
                }
#pragma unroll
                for (int r = 0; r < R; ++r) a[j][r] = ldw(cn + cr[r]);
                __builtin_amdgcn_sched_barrier(0);
            }
            end_stage();
            buf ^= 1;
        }
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
                for (int t = 0; t < TW; ++t) {
                    const int tok = 16 * (t_off + t) + tok_l;
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
        __shared__ float s_val[WN][T * 16];
        __shared__ int s_idx[WN][T * 16];
#pragma unroll
        for (int t = 0; t < TW; ++t) {
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
                s_val[wave_n][16 * (t_off + t) + lane] = best;
                s_idx[wave_n][16 * (t_off + t) + lane] = bidx;
            }
        }
        __syncthreads();
        const int tok = threadIdx.x;
        if (tok < T * 16 && tok < m_rows) {
            float best = s_val[0][tok];
            int bidx = s_idx[0][tok];
            for (int w = 1; w < WN; ++w) {
                const float ov = s_val[w][tok];
                const int oi = s_idx[w][tok];
                if (ov > best || (ov == best && oi < bidx)) { best = ov; bidx = oi; }
            }
            g.arg_val[(size_t)(pass * 16 * T + tok) * g.arg_groups + bx] = best;
            g.arg_idx[(size_t)(pass * 16 * T + tok) * g.arg_groups + bx] = bidx;
        }
    }
    if (EPI == EPI_SWIGLU) {  // even tiles are gate rows, odd tiles the matching up rows
#pragma unroll
        for (int p = 0; p < R / 2; ++p) {
            const int j = (((nt0 >> 1) + p) * 16) + n_l;
            if (j >= g.ffn) break;
#pragma unroll
            for (int t = 0; t < TW; ++t) {
                const int tok = 16 * (t_off + t) + tok_l;
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
#endif
}

template <int W, int R, int EPI>
hipError_t launch_wide_r(const GemmLaunch& g, int ksplit, int n_groups, int kt_per_split, hipStream_t s) {
    constexpr int T = kWideRowTiles, KS = kWideStage;
    const dim3 grid(8 * ceil_div(n_groups * ksplit, 8) * g.passes), block(64 * W);
    hipLaunchKernelGGL((gemm_wide_kernel<W, kWideRowSplit, R, T, KS, kWideDepth, kWideTB, EPI>), grid, block, 0, s, g, ksplit, n_groups,
                       kt_per_split);
    return hipGetLastError();
}

}  // namespace

WidePlan plan_gemm_wide(const PackedW& w, int m, GemmEpilogue epi, int max_splits) {
    WidePlan p{};
    p.passes = ceil_div(m, 16 * kWideRowTiles);
    p.tiles_per_wave = kWideTiles;
    p.n_groups = ceil_div(w.n_tiles, kWideWaves / kWideRowSplit * kWideTiles);
    // Split of the contraction (plain sums only): a CU works through its share of the workgroups at a
    // rate that hardly depends on how many it holds at once, so the time goes with
    // ceil(workgroups / CUs) * contraction tiles per workgroup; every doubling costs a little for the
    // partial sums, and a split keeps at least 16 tiles.
    const int smax = (epi == EPI_F32) ? (max_splits < 4 ? max_splits : 4) : 1;
    double best = 1e30;
    p.ksplit = 1;
    for (int ks = 1; ks <= smax; ks *= 2) {
        if (ks > 1 && w.k_tiles / ks < 16) break;
        const double cost = (double)ceil_div(p.n_groups * p.passes * ks, 256) * ceil_div(w.k_tiles, ks) * (ks == 1 ? 1.0 : ks == 2 ? 1.04 : 1.08);
        if (cost < best) { best = cost; p.ksplit = ks; }
    }
    p.kt_per_split = round_up(ceil_div(w.k_tiles, p.ksplit), kWideDepth);
    p.ksplit = ceil_div(w.k_tiles, p.kt_per_split);  // no empty split
    return p;
}

hipError_t launch_gemm_wide(const GemmLaunch& g0, const WidePlan& p, GemmEpilogue epi, hipStream_t s) {
    GemmLaunch g = g0;
    g.passes = p.passes;
    if (g.m < 1 || p.passes != ceil_div(g.m, 16 * kWideRowTiles) || g.row_tile0 != 0 || g.w.k_tiles < 1 ||
        g.xs.row_tiles != ceil_div(g.m, 16) || g.xs.last_cols != g.m - 16 * (g.xs.row_tiles - 1))
        return hipErrorInvalidValue;
    if (p.ksplit < 1 || p.kt_per_split < 1 || p.kt_per_split % kWideDepth || (p.ksplit - 1) * p.kt_per_split >= g.w.k_tiles ||
        p.ksplit * p.kt_per_split < g.w.k_tiles || round_up(g.w.k_tiles, kWideDepth) > g.w.k_tiles_pad() ||
        p.n_groups != ceil_div(g.w.n_tiles, kWideWaves / kWideRowSplit * p.tiles_per_wave))
        return hipErrorInvalidValue;
    if (epi != EPI_F32 && p.ksplit != 1) return hipErrorInvalidValue;
    if (g.w.bytes() >= ((size_t)1 << 32)) return hipErrorInvalidValue;  // the kernel addresses the matrix with 32-bit byte offsets
    if (epi == EPI_ARGMAX && p.n_groups > g.arg_groups) return hipErrorInvalidValue;
#define SPACE_WIDE(RR)                                                                                                     \
    switch (epi) {                                                                                                         \
        case EPI_F32: return launch_wide_r<kWideWaves, RR, EPI_F32>(g, p.ksplit, p.n_groups, p.kt_per_split, s);           \
        case EPI_SWIGLU: return launch_wide_r<kWideWaves, RR, EPI_SWIGLU>(g, p.ksplit, p.n_groups, p.kt_per_split, s);     \
        case EPI_ARGMAX: return launch_wide_r<kWideWaves, RR, EPI_ARGMAX>(g, p.ksplit, p.n_groups, p.kt_per_split, s);     \
    }
    if (p.tiles_per_wave == kWideTiles) { SPACE_WIDE(kWideTiles) }
#undef SPACE_WIDE
    return hipErrorInvalidValue;
}

}  // namespace space
