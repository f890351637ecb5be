// bf16 MFMA GEMM for gfx950:  C = A[M][K] * W[N][K]^T, fp32 accumulation.
//
// Both operands are K-contiguous, which is what the 32x32x16 bf16 MFMA wants: a
// lane feeds 8 consecutive K values of one row (A) or one column (W).  A
// workgroup of four waves (2x2 or 4x1, one wave per SIMD) owns a BM x BN tile
// and walks K in stages of BK = 32 or 64 through an LDS ring of NST stages.
// Large wave tiles (up to 128x128) keep the LDS fragment traffic per flop low:
// under MFMA load the chip is power limited (measured shader clocks of 1.4 to
// 1.8 GHz), so bytes moved per flop decide the sustained rate as much as issue
// slots do.
//
// Main kernel (gemm_il_kernel, K % 64 == 0):
//   * global -> LDS copies are asynchronous (global_load_lds_dwordx4, 1 KB per
//     wave instruction, no VGPR staging) and run NST-1 stages ahead of the math.
//   * One wave per SIMD means nothing else fills an issue bubble, so the stream
//     is software-pipelined by hand: the fragment reads for the next K-substep
//     and the copies of a later stage are spread one by one between the MFMAs
//     of the current substep (an LDS read or copy issued right after an MFMA
//     costs nothing, a clump of them stalls the matrix pipe), and the only
//     barrier of a stage sits in front of the last substep's MFMAs, which hide
//     it together with the first fragment reads of the next stage.
//   * The loop is split into a steady state (every step issues copies) and a
//     tail (none left), so there is no branch between MFMAs; wait counts are
//     compile-time constants in the steady state.
//   * LDS rows are BK*2 bytes; 16-byte chunks are XOR-swizzled ((row >> 1) & 7
//     for 128-byte rows, (row >> 2) & 3 for 64-byte rows): the LDS has 64 banks
//     and serves 16 lanes x 16 bytes per cycle, and this keeps each such group
//     of fragment reads on 64 distinct banks.  The swizzle is applied by
//     choosing which global chunk each lane copies, because the LDS side of the
//     copy is fixed (lane * 16 bytes).
//   * MFMAs are issued as (W fragment) x (A fragment): the accumulators then hold
//     the transposed tile, four consecutive output columns per lane, and the
//     epilogue stores 8 (bf16) or 16 (fp32) bytes per lane.
//   * Every kernel argument is forced into registers before the loop: a scalar
//     load still pending at the loop header shares its counter with the LDS
//     reads and would make the compiler wait for all of them at every use.
// Fallback kernel (gemm_reg_kernel): any K % 8 == 0, register-staged loads with
// zero fill, two LDS stages.
//
// Epilogues: bf16 store; fp32 slabs for split-K, which the next residual-add +
// RMSNorm kernel sums; row statistics (maximum, sum of exponentials and arg max
// of every row over each wave's column slice: the greedy decode of Section 3.1
// eq. 3 on the vocabulary projection, which then writes no logits); and two
// "paired" epilogues, SwiGLU and rotary embedding, that combine two output columns.  For those the W rows of a tile are permuted
// while they are copied: every 32-row MFMA tile holds 16 first partners (gate
// rows; first half of a head) followed by their 16 second partners (up rows;
// second half of the head), so both values of a pair end up in the same lane,
// 8 accumulator elements apart, whatever the wave layout.
//
// Workgroup ids are mapped so that the tiles sharing a weight column block run on
// the same XCD (ids congruent mod 8 share an L2), and the workgroups of an XCD that
// run together cover a few row tiles times a few column tiles (see tile_of).
#include <stdio.h>
#include <stdlib.h>

#include <map>
#include <mutex>
#include <tuple>
#include <type_traits>

#include "internal.h"

namespace dllm {

namespace {

#define DLLM_LDS_VOID(p) ((__attribute__((address_space(3))) void *)(p))

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v)
{
    union { uint4 u; bf16x8 b; } c;
    c.u = v;
    return c.b;
}

// Asynchronous 16-byte-per-lane global -> LDS copy; LDS address = m0 + lane * 16.
// Inline asm on purpose: with the compiler builtin every later LDS read is
// preceded by a conservative "s_waitcnt vmcnt(0)", which serialises the copy of
// the next K-steps with the math on the current one.  Waits are placed by hand.
// NT: the non-temporal hint, for bytes that are read once (the vocabulary projection's weights under a single
// row tile): a copy-only probe streams 27.5 instead of 24.4 GB/s per CU from HBM with it.
template <bool NT = false>
__device__ __forceinline__ void async_load16(const char *base_uniform, uint32_t voffset, uint32_t lds_addr_uniform)
{
    if constexpr (NT)
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 nt"
                     :
                     : "s"(lds_addr_uniform), "v"(voffset), "s"(base_uniform)
                     : "memory");
    else
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                     :
                     : "s"(lds_addr_uniform), "v"(voffset), "s"(base_uniform)
                     : "memory");
}
__device__ __forceinline__ uint32_t lds_addr_of(const void *p)
{
    return __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)DLLM_LDS_VOID(p));
}
template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
// at most n * LOADS copies may still be in flight, n in [0, MAXN]
template <int MAXN, int LOADS>
__device__ __forceinline__ void wait_stages_after(int n)
{
    if constexpr (MAXN <= 0) {
        wait_vmcnt<0>();
    } else {
        if (n >= MAXN) wait_vmcnt<(MAXN * LOADS > 63 ? 63 : MAXN * LOADS)>();
        else wait_stages_after<MAXN - 1, LOADS>(n);
    }
}

// tile of this workgroup; tiles that share W rows get ids congruent mod 8 (the same XCD, one L2).
// Inside an XCD the workgroups that run together (consecutive local ids) cover kGroupM row tiles
// times a few column tiles, so that the L2 serves few distinct A and W slices at a time (with two
// row tiles, M = 512, this is "all row tiles of a column tile, then the next column tile").
constexpr int kGroupM = 4;
__device__ __forceinline__ void tile_of(int pid, int num_m, int num_n, int &pid_m, int &pid_n)
{
    const int n8 = num_n & ~7, head = num_m * n8;
    if (pid < head) {
        const int xcd = pid & 7, j = pid >> 3, nt = n8 >> 3;  // local id; column tiles of this XCD
        const int in_group = kGroupM * nt, group = j / in_group, r = j - group * in_group;
        const int first_m = group * kGroupM, gm = min(num_m - first_m, kGroupM);
        pid_m = first_m + r % gm;
        pid_n = (r / gm) * 8 + xcd;
    } else {
        const int r = pid - head;
        pid_m = r % num_m;
        pid_n = n8 + r / num_m;
    }
}

// Rotary embedding fused into the QKV projection's epilogue: output columns
// below rope_cols (the q and k thirds) are rotated in fp32 before the bf16
// rounding; pos = row % L, table[pos][j] = (cos, sin) of pos * theta^(-2j/dh).
//
// The row-statistics epilogue (greedy decode and confidence of Section 3.1 eq. 3 taken on the
// accumulators of the vocabulary projection, so that the logits are never written) reuses the two
// integers: `parts` column slices per row (one per wave column of every tile) and the id of the
// [MASK] token, which is not a legal prediction.
struct RopeArgs {
    const float2 *table;
    const int32_t *pos;  // nullable: position of every row (rows of a gathered subset)
    union { int L; int parts; };
    union { int rope_cols; int mask_id; };
    // Operand layouts (see GemmLayout): byte distance between consecutive rows and between consecutive
    // 32-element K panels of A and of W, and the panel rows of a panel-major SwiGLU output (0: row-major).
    uint32_t a_row_pitch, a_panel_pitch, w_row_pitch, w_panel_pitch;
    int c_panel_rows;
    // RMSNorm folded into the product that consumes the normalised rows (see RowScale): every output row r is
    // scaled by rsqrt(sum_p row_ssq[r * ssq_stride + p] / K + eps) before its epilogue.  Null: no scaling.
    const float *row_ssq;
    int ssq_parts, ssq_stride;
    float eps;
    // Residual epilogue (see ResidualOut); Cout then holds the fp32 split-K slabs.
    // (the rotary epilogues use two of its fields for their own purpose: with kv_dst set, the K and V thirds of
    // output row r go to row kv_rows[r] of kv_dst, a [rows][3 d] array, instead of row r of Cout)
    float *x;
    const uint16_t *gain;
    union { uint16_t *h_out; uint16_t *kv_dst; };
    float *ssq_out;
    union { int *tickets; const int32_t *kv_rows; };
    int ssq_out_stride;
};
constexpr int kEpiRope64 = 3, kEpiRope128 = 4;  // head_dim is a compile-time constant of the epilogue
constexpr int kEpiRowStats = 5;
constexpr int kEpiResidual = 6;  // the O and down projections: see residual_tile

__host__ __device__ constexpr bool epi_paired(int epi) { return epi == kEpiSwiglu || epi == kEpiRope64 || epi == kEpiRope128; }
__host__ __device__ constexpr int epi_head_dim(int epi) { return epi == kEpiRope128 ? 128 : 64; }

// Global W row held by row j of a workgroup's W tile.  Plain epilogues: n0 + j.
// Paired epilogues: the tile covers pairs [pair0, pair0 + BN/2); MFMA tile s =
// j / 32 holds pairs pair0 + 16 s .. + 15, first partners in its rows 0..15,
// second partners in rows 16..31.  n_pairs = number of pairs of the whole
// matrix (SwiGLU: features, the up row of feature p is n_pairs + p; rotary:
// columns c and c + dh/2 of a head).  Rows past the edge are clamped.
template <int EPI>
__device__ __forceinline__ int w_global_row(int j, int n0, int N)
{
    if (!epi_paired(EPI)) return min(n0 + j, N - 1);
    const int n_pairs = N / 2;
    const int p = min(n0 + (j >> 5) * 16 + (j & 15), n_pairs - 1), second = (j >> 4) & 1;
    if (EPI == kEpiSwiglu) return second * n_pairs + p;
    constexpr int HD = epi_head_dim(EPI) / 2;
    return (p / HD) * (2 * HD) + second * HD + p % HD;
}

// Accumulators hold the transposed 32x32 tiles: element e of lane l is output
// row l % 32, tile column 8*(e/4) + 4*(l/32) + e%4.  n0 is the first output
// column (plain) or the first pair (paired) of the workgroup's tile.
// GUARD = false: the workgroup's tile lies inside the matrix and N % 4 == 0, so no store needs a
// bounds check (straight-line stores with immediate offsets instead of a masked branch per store).
// s_inv (LDS, nullable): per row of the workgroup's tile, the factor every accumulator of that row is
// multiplied with where the epilogue reads it (the RMSNorm of the rows that were multiplied, see RowScale).
template <int TM, int TN, int WTM, int EPI, bool GUARD>
__device__ __forceinline__ void store_tile(floatx16 (&acc)[TM][TN], void *Cout, int M, int N, int m0, int n0, int wm,
                                           int wn, int l32, int lhalf, int split, const RopeArgs &rope,
                                           const float *s_inv = nullptr)
{
    if constexpr (EPI == kEpiRowStats) {
        // Cout: fp32 max [parts][M], fp32 sum of exp(x - max) [parts][M], int32 lowest column of the max
        // [parts][M]; x = the logit rounded to bf16 (what the unfused path stores and reads back); the
        // slice of this wave is part n0 / (32 TN) + wn.  A slice without a legal column leaves (-3e38, 0).
        constexpr float kLog2e = 1.4426950408889634f, kNegBig = -3.0e38f;
        const size_t plane = (size_t)rope.parts * M;
        float *pm = reinterpret_cast<float *>(Cout) + (size_t)(n0 / (32 * TN) + wn) * M;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int row = m0 + wm * WTM + i * 32 + l32;
            const float inv = s_inv ? s_inv[wm * WTM + i * 32 + l32] : 1.0f;
            float m = kNegBig;
            int c = 0x7fffffff;
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int col = n0 + (wn * TN + j) * 32 + 8 * q + 4 * lhalf;
                    const uint32_t w01 = pack_bf16x2(acc[i][j][4 * q] * inv, acc[i][j][4 * q + 1] * inv);
                    const uint32_t w23 = pack_bf16x2(acc[i][j][4 * q + 2] * inv, acc[i][j][4 * q + 3] * inv);
                    const float x[4] = {__uint_as_float(w01 << 16), __uint_as_float(w01 & 0xffff0000u),
                                        __uint_as_float(w23 << 16), __uint_as_float(w23 & 0xffff0000u)};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const bool legal = col + e < N && col + e != rope.mask_id;
                        const float v = legal ? x[e] : -INFINITY;
                        acc[i][j][4 * q + e] = v;
                        if (v > m) {  // columns are visited in increasing order: the first maximum stays
                            m = v;
                            c = col + e;
                        }
                    }
                }
            const float off = -m * kLog2e;
            float s = 0.0f;
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) s += __builtin_amdgcn_exp2f(fmaf(acc[i][j][e], kLog2e, off));
            s = m > kNegBig ? s : 0.0f;
            // the other half of the row's columns sits in lane ^ 32
            const float m2 = __shfl_xor(m, 32, 64), s2 = __shfl_xor(s, 32, 64);
            const int c2 = __shfl_xor(c, 32, 64);
            const float mt = fmaxf(m, m2);
            const float st = s * __builtin_amdgcn_exp2f((m - mt) * kLog2e) + s2 * __builtin_amdgcn_exp2f((m2 - mt) * kLog2e);
            const int ct = (m > m2 || (m == m2 && c < c2)) ? c : c2;
            if (lhalf == 0 && row < M) {
                pm[row] = mt;
                pm[plane + row] = st;
                reinterpret_cast<int *>(pm)[2 * plane + row] = ct;
            }
        }
    } else if (EPI == kEpiSwiglu) {
        uint16_t *C = reinterpret_cast<uint16_t *>(Cout);
        const int n_out = N / 2;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int row = m0 + wm * WTM + i * 32 + l32;
            const float inv = s_inv ? s_inv[wm * WTM + i * 32 + l32] : 1.0f;
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    const int col = n0 + (wn * TN + j) * 16 + 8 * q + 4 * lhalf;
                    float y[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float g = acc[i][j][4 * q + e] * inv, u = acc[i][j][8 + 4 * q + e] * inv;
                        y[e] = g * __builtin_amdgcn_rcpf(1.0f + __expf(-g)) * u;  // 1 ulp reciprocal, far below the bf16 rounding
                    }
                    if (GUARD && (row >= M || col >= n_out)) continue;
                    // panel-major: element (row, col) sits at ((col / 32) * panel_rows + row) * 32 + col % 32
                    uint16_t *p = rope.c_panel_rows
                                      ? C + ((size_t)(col >> 5) * rope.c_panel_rows + row) * 32 + (col & 31)
                                      : C + (size_t)row * n_out + col;
                    if (!GUARD || (col + 3 < n_out && (n_out & 3) == 0)) {
                        uint2 w;
                        w.x = pack_bf16x2(y[0], y[1]);
                        w.y = pack_bf16x2(y[2], y[3]);
                        *reinterpret_cast<uint2 *>(p) = w;
                    } else {
                        for (int e = 0; e < 4 && col + e < n_out; ++e) p[e] = float_to_bf16_bits(y[e]);
                    }
                }
        }
    } else if (EPI == kEpiRope64 || EPI == kEpiRope128) {
        // N % head_dim == 0 and head_dim % 32 == 0 (checked by the host): the 4 pairs of a lane
        // share a head, and whole 16-byte groups are inside or outside the matrix
        constexpr int HD = epi_head_dim(EPI) / 2;
        uint16_t *C = reinterpret_cast<uint16_t *>(Cout);
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int row = m0 + wm * WTM + i * 32 + l32;
            const float2 *trow = rope.table + (size_t)(rope.pos ? rope.pos[min(row, M - 1)] : row % rope.L) * HD;
            const float inv = s_inv ? s_inv[wm * WTM + i * 32 + l32] : 1.0f;
            // keys and values of a gathered row go straight to the row's place in the cache
            uint16_t *crow = C + (size_t)row * N;
            uint16_t *kvrow = rope.kv_dst ? rope.kv_dst + (size_t)rope.kv_rows[min(row, M - 1)] * N : crow;
            const int kv_first = N / 3;
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    const int p = n0 + (wn * TN + j) * 16 + 8 * q + 4 * lhalf;  // first of the lane's 4 pairs
                    const int pp = p % HD, col = (p / HD) * (2 * HD) + pp;
                    if (GUARD && (row >= M || p >= N / 2)) continue;
                    float a[4], b[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        a[e] = acc[i][j][4 * q + e] * inv;
                        b[e] = acc[i][j][8 + 4 * q + e] * inv;
                    }
                    if (col < rope.rope_cols) {
                        const float4 *tp = reinterpret_cast<const float4 *>(trow + pp);  // 4 (cos, sin) pairs
                        const float4 t01 = tp[0], t23 = tp[1];
                        const float cs[4] = {t01.x, t01.z, t23.x, t23.z}, sn[4] = {t01.y, t01.w, t23.y, t23.w};
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float x = a[e], y = b[e];
                            a[e] = x * cs[e] - y * sn[e];
                            b[e] = x * sn[e] + y * cs[e];
                        }
                    }
                    uint16_t *dst = (col >= kv_first ? kvrow : crow) + col;   // (a pair never straddles two thirds)
                    uint2 w;
                    w.x = pack_bf16x2(a[0], a[1]);
                    w.y = pack_bf16x2(a[2], a[3]);
                    *reinterpret_cast<uint2 *>(dst) = w;
                    w.x = pack_bf16x2(b[0], b[1]);
                    w.y = pack_bf16x2(b[2], b[3]);
                    *reinterpret_cast<uint2 *>(dst + HD) = w;
                }
        }
    } else if (EPI == kEpiBf16) {
        uint16_t *C = reinterpret_cast<uint16_t *>(Cout);
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int row = m0 + wm * WTM + i * 32 + l32;
            const float inv = s_inv ? s_inv[wm * WTM + i * 32 + l32] : 1.0f;
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int col = n0 + (wn * TN + j) * 32 + 8 * q + 4 * lhalf;
                    if (GUARD && (row >= M || col >= N)) continue;
                    uint16_t *p = C + (size_t)row * N + col;
                    if (!GUARD || (col + 3 < N && (N & 3) == 0)) {
                        uint2 w;
                        w.x = pack_bf16x2(acc[i][j][4 * q] * inv, acc[i][j][4 * q + 1] * inv);
                        w.y = pack_bf16x2(acc[i][j][4 * q + 2] * inv, acc[i][j][4 * q + 3] * inv);
                        *reinterpret_cast<uint2 *>(p) = w;
                    } else {
                        for (int e = 0; e < 4 && col + e < N; ++e) p[e] = float_to_bf16_bits(acc[i][j][4 * q + e] * inv);
                    }
                }
        }
    } else {
        float *C = reinterpret_cast<float *>(Cout) + (size_t)split * M * N;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int row = m0 + wm * WTM + i * 32 + l32;
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int col = n0 + (wn * TN + j) * 32 + 8 * q + 4 * lhalf;
                    if (GUARD && (row >= M || col >= N)) continue;
                    float *p = C + (size_t)row * N + col;
                    if (!GUARD || (col + 3 < N && (N & 3) == 0)) {
                        *reinterpret_cast<float4 *>(p) = make_float4(acc[i][j][4 * q], acc[i][j][4 * q + 1],
                                                                     acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
                    } else {
                        for (int e = 0; e < 4 && col + e < N; ++e) p[e] = acc[i][j][4 * q + e];
                    }
                }
        }
    }
}

// Residual epilogue of the O and down projections.  The workgroup that runs it holds the tile's last
// missing partial product in its accumulators; the other K splits' partial tiles are in the slabs.
//   x[row][col] += partial_0 + partial_1 + ...        (fp32 residual stream, in split order)
//   h_out[row][col] = bf16(x[row][col] * gain[col])   (operand of the next projection, not yet normalised:
//                                                      that product scales its rows, see RowScale)
//   ssq_out[row][part] = sum over this wave's columns of x[row][col]^2, part = (column tile, wave column)
// FROM_SLABS = false: one K split, the accumulators are the whole product.  FROM_SLABS = true: every split's
// partial tile (this workgroup's too) is read back from the slabs and added in split order, so the sum does
// not depend on which split came last.
template <int TM, int TN, int WTM, bool FROM_SLABS>
__device__ __forceinline__ void residual_tile(floatx16 (&acc)[TM][TN], const float *slabs, int splits, int M, int N, int m0,
                                              int n0, int wm, int wn, int l32, int lhalf, int part, const RopeArgs &ea)
{
    const size_t slab = (size_t)M * N;
    constexpr int NV = TN * 4;              // float4 positions of a lane in one 32-row block
    // handled at a time (a divisor of NV): the widest tiles have no registers for more
    constexpr int NC = NV <= 8 ? NV : NV % 8 == 0 ? 8 : NV % 6 == 0 ? 6 : 4;
    static_assert(NV % NC == 0, "whole chunks");
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int row = m0 + wm * WTM + i * 32 + l32;
        float ss = 0.0f;
#pragma unroll
        for (int c0 = 0; c0 < NV; c0 += NC) {
            float4 v[NC];
            bool ok[NC];
#pragma unroll
            for (int u = 0; u < NC; ++u) {
                const int jq = c0 + u;
                const int col = n0 + (wn * TN + jq / 4) * 32 + 8 * (jq % 4) + 4 * lhalf;
                ok[u] = row < M && col < N;                       // (N % 4 == 0: checked by the host)
                v[u] = ok[u] ? *reinterpret_cast<const float4 *>(ea.x + (size_t)row * N + col) : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            }
            if constexpr (FROM_SLABS) {
                for (int s = 0; s < splits; ++s) {
                    float4 p[NC];
#pragma unroll
                    for (int u = 0; u < NC; ++u) {
                        const int jq = c0 + u;
                        const int col = n0 + (wn * TN + jq / 4) * 32 + 8 * (jq % 4) + 4 * lhalf;
                        p[u] = ok[u] ? *reinterpret_cast<const float4 *>(slabs + s * slab + (size_t)row * N + col)
                                     : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
                    }
#pragma unroll
                    for (int u = 0; u < NC; ++u) { v[u].x += p[u].x; v[u].y += p[u].y; v[u].z += p[u].z; v[u].w += p[u].w; }
                }
            } else {
#pragma unroll
                for (int u = 0; u < NC; ++u) {
                    const int j = (c0 + u) / 4, q = (c0 + u) % 4;
                    v[u].x += acc[i][j][4 * q]; v[u].y += acc[i][j][4 * q + 1]; v[u].z += acc[i][j][4 * q + 2]; v[u].w += acc[i][j][4 * q + 3];
                }
            }
#pragma unroll
            for (int u = 0; u < NC; ++u) {
                if (!ok[u]) continue;
                const int jq = c0 + u;
                const int col = n0 + (wn * TN + jq / 4) * 32 + 8 * (jq % 4) + 4 * lhalf;
                const size_t at = (size_t)row * N + col;
                const float4 t = v[u];
                *reinterpret_cast<float4 *>(ea.x + at) = t;
                ss += t.x * t.x + t.y * t.y + t.z * t.z + t.w * t.w;
                const uint2 g = *reinterpret_cast<const uint2 *>(ea.gain + col);
                uint2 o;
                o.x = pack_bf16x2(t.x * bf16_lo(g.x), t.y * bf16_hi(g.x));
                o.y = pack_bf16x2(t.z * bf16_lo(g.y), t.w * bf16_hi(g.y));
                uint16_t *hp = ea.c_panel_rows ? ea.h_out + ((size_t)(col >> 5) * ea.c_panel_rows + row) * 32 + (col & 31)
                                               : ea.h_out + at;
                *reinterpret_cast<uint2 *>(hp) = o;
            }
        }
        ss += __shfl_xor(ss, 32, 64);                               // the other half of the row's columns
        if (lhalf == 0 && row < M) ea.ssq_out[(size_t)row * ea.ssq_out_stride + part] = ss;
    }
}

// The tail of a kEpiResidual workgroup: with one K split the accumulators are the whole product; with more,
// every split leaves its partial tile in its slab and takes a ticket, and the split that takes the last ticket
// of a tile adds everything up (the others are done).  No workgroup waits for another.
template <int TM, int TN, int WTM, int WN>
__device__ __forceinline__ void residual_finish(floatx16 (&acc)[TM][TN], void *slabs, int M, int N, int m0, int n0, int wm,
                                                int wn, int l32, int lhalf, int pid_n, const RopeArgs &ea)
{
    __shared__ int s_ticket;
    const int splits = gridDim.y, my_split = blockIdx.y;
    if (splits > 1) {
        store_tile<TM, TN, WTM, kEpiPartial, true>(acc, slabs, M, N, m0, n0, wm, wn, l32, lhalf, my_split, ea);
        // One thread publishes for the workgroup: the barrier orders every thread's slab stores before its
        // device-scope release (a single write-back of the L2 per workgroup instead of one per wave), the
        // ticket is taken, and only the workgroup that finds itself last pays for the acquire (which drops
        // what its L2 holds of other workgroups' lines).  The second barrier hands the result to the others.
        __syncthreads();
        if (threadIdx.x == 0) {
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
            const int t = __hip_atomic_fetch_add(&ea.tickets[blockIdx.x], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (t == splits - 1) {
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
                ea.tickets[blockIdx.x] = 0;    // ready for the next launch; nobody else looks at it any more
            }
            s_ticket = t;
        }
        __syncthreads();
        if (s_ticket != splits - 1) return;    // uniform over the workgroup
    }
    if (splits > 1)
        residual_tile<TM, TN, WTM, true>(acc, reinterpret_cast<const float *>(slabs), splits, M, N, m0, n0, wm, wn, l32, lhalf,
                                         pid_n * WN + wn, ea);
    else
        residual_tile<TM, TN, WTM, false>(acc, nullptr, 1, M, N, m0, n0, wm, wn, l32, lhalf, pid_n * WN + wn, ea);
}

// RowScale: the factors of the workgroup's BM rows, rsqrt(mean square + eps) from the partial sums of squares
// that the producer of the rows left (embedding kernel or a residual epilogue), summed in part order.
template <int BM>
__device__ __forceinline__ void row_scale_prologue(float *s_inv, int m0, int M, int K, const RopeArgs &ea)
{
    if (!ea.row_ssq) return;
    for (int t = threadIdx.x; t < BM; t += blockDim.x) {
        const float *p = ea.row_ssq + (size_t)min(m0 + t, M - 1) * ea.ssq_stride;
        float sum = 0.0f;
        if (((ea.ssq_parts | ea.ssq_stride) & 3) == 0) {   // rows of whole, aligned float4
            const float4 *p4 = reinterpret_cast<const float4 *>(p);
            const int n4 = ea.ssq_parts >> 2;
            for (int k0 = 0; k0 < n4; k0 += 8) {           // eight loads in flight, summed in part order
                float4 v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) v[u] = k0 + u < n4 ? p4[k0 + u] : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
#pragma unroll
                for (int u = 0; u < 8; ++u) sum += (v[u].x + v[u].y) + (v[u].z + v[u].w);
            }
        } else {
            for (int k = 0; k < ea.ssq_parts; ++k) sum += p[k];
        }
        s_inv[t] = rsqrtf(sum / (float)K + ea.eps);
    }
}

// ---- main kernel: K % BK == 0, k_per_split % BK == 0 ---------------------------
template <int BM, int BN, int WM, int WN, int BK, int NST, int EPI>
__global__ __launch_bounds__(WM * WN * 64) void gemm_il_kernel(const uint16_t *__restrict__ A,
                                                           const uint16_t *__restrict__ W, void *__restrict__ Cout,
                                                           int M, int N, int K, int k_per_split, int num_m, int num_n,
                                                           RopeArgs rope)
{
    constexpr int NW = WM * WN;
    constexpr int WTM = BM / WM, WTN = BN / WN, TM = WTM / 32, TN = WTN / 32;
    static_assert(TM >= 1 && TN >= 1 && WTM % 32 == 0 && WTN % 32 == 0, "wave tile is made of 32x32 MFMA tiles");
    static_assert(BK == 32 || BK == 64, "stage depth");
    // 16-byte chunks per LDS row, K-substeps per stage, rows moved by one copy instruction of a wave
    constexpr int CPR = BK / 8, KS = BK / 16, RPI = 64 / CPR;
    constexpr int ROWS = BM + BN;  // rows of one stage: the A tile, then the W tile
    constexpr int NI = ROWS / RPI, LOADS = NI / NW, A_NI = BM / RPI;
    static_assert(ROWS % RPI == 0 && NI % NW == 0 && BM % RPI == 0, "whole copy instructions per wave");
    constexpr bool kNtW = EPI == kEpiRowStats && A_NI % NW == 0;   // (copy t of a wave moves W rows iff t >= A_NI / NW)
    constexpr int P = NST - 1;  // stages in flight ahead of the one being multiplied
    static_assert(NST >= 3, "the stage after the current one is completely issued one step ahead");
    static_assert(P * LOADS <= 63, "outstanding copies fit the wait counter");
    constexpr int STAGE = ROWS * CPR;  // uint4 per stage
    constexpr int NMF = TM * TN, NRD = TM + TN;
    extern __shared__ uint4 smem[];

    int pid_m, pid_n;
    tile_of(blockIdx.x, num_m, num_n, pid_m, pid_n);
    constexpr int BN_OUT = epi_paired(EPI) ? BN / 2 : BN;  // output columns (plain) or pairs (paired) per tile
    const int m0 = pid_m * BM, n0 = pid_n * BN_OUT;
    const int kbeg = blockIdx.y * k_per_split;
    const int kend = min(K, kbeg + k_per_split);
    const int nk = (kend - kbeg) / BK;

    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int wm = wave / WN, wn = wave % WN;
    const int l32 = lane & 31, lhalf = lane >> 5;

    // copy instruction q = wave + NW * t moves LDS rows [q * RPI, (q + 1) * RPI); lane l lands on row
    // l / CPR, slot l % CPR of that group and therefore fetches the chunk that the swizzle puts there
    // An operand is row-major (row pitch = K * 2 bytes, the 32-element K panels of a row follow each
    // other: panel pitch 64) or panel-major (panel p holds elements [32 p, 32 p + 32) of every row: row pitch
    // 64, panel pitch = rows * 64).  Chunk c of a stage's row (16 bytes each) is in panel c / 4, at c % 4.
    const int lrow = lane / CPR, lslot = lane % CPR;
    uint32_t goff[LOADS];  // byte offsets into A or W; rows past the edge are clamped
#pragma unroll
    for (int t = 0; t < LOADS; ++t) {
        const int q = wave + NW * t, r = q * RPI + lrow;
        const int swz = BK == 64 ? ((r >> 1) & 7) : ((r >> 2) & 3);
        const int grow = q < A_NI ? min(m0 + r, M - 1) : w_global_row<EPI>(r - BM, n0, N);
        const int chunk = lslot ^ swz;
        const uint32_t row_pitch = q < A_NI ? rope.a_row_pitch : rope.w_row_pitch;
        const uint32_t panel_pitch = q < A_NI ? rope.a_panel_pitch : rope.w_panel_pitch;
        goff[t] = (uint32_t)grow * row_pitch + (uint32_t)(chunk >> 2) * panel_pitch + (chunk & 3) * 16;
    }
    const size_t a_stage = (size_t)(BK / 32) * rope.a_panel_pitch, w_stage = (size_t)(BK / 32) * rope.w_panel_pitch;
    const char *Ab = reinterpret_cast<const char *>(A) + (size_t)(kbeg / 32) * rope.a_panel_pitch;
    const char *Wb = reinterpret_cast<const char *>(W) + (size_t)(kbeg / 32) * rope.w_panel_pitch;
    const uint32_t lds0 = lds_addr_of(smem) + wave * 1024;
#define DLLM_COPY(t_, stage_, slot_)                                                             \
    do {                                                                                         \
        const bool a_ = (wave + NW * (t_)) < A_NI;                                               \
        const char *b_ = (a_ ? Ab : Wb) + (size_t)(stage_) * (a_ ? a_stage : w_stage);           \
        if (kNtW && (t_) >= A_NI / NW) async_load16<true>(b_, goff[t_], lds0 + (slot_) * (STAGE * 16) + (t_) * (NW * 1024)); \
        else async_load16<false>(b_, goff[t_], lds0 + (slot_) * (STAGE * 16) + (t_) * (NW * 1024)); \
    } while (0)

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    const int sw = BK == 64 ? ((l32 >> 1) & 7) : ((l32 >> 2) & 3);
    const int a_base = (wm * WTM + l32) * CPR, b_base = (BM + wn * WTN + l32) * CPR;  // uint4 index of fragment 0's row
    // 32-row sub-tiles of this wave that hold at least one real row: the MFMAs of the others are
    // skipped (a ragged last M tile then costs its workgroups only the copies, and the chip is
    // power limited, so the cycles and the energy go to the tiles that have rows)
    // (not in the 256x256 tile, whose 256 accumulator registers leave no room for one more value)
    constexpr bool kSkipEmpty = BM * BN < 256 * 256;
    constexpr bool kEarlyReads = true;
    const int tm_valid = kSkipEmpty ? __builtin_amdgcn_readfirstlane(min(TM, max(0, (M - m0 - wm * WTM + 31) / 32))) : TM;
    bf16x8 af[2][TM], bfr[2][TN];
    // fragments are read in the order of their first use by the MFMA sequence (i outer, j inner):
    // A0, W0 .. W(TN-1), A1 .. A(TM-1)
#define DLLM_READ(ridx_, st_, ch_, buf_)                                                                  \
    do {                                                                                                  \
        if ((ridx_) == 0) af[buf_][0] = as_bf16x8((st_)[a_base + (ch_)]);                                 \
        else if ((ridx_) <= TN) bfr[buf_][((ridx_) - 1) % TN] = as_bf16x8((st_)[b_base + ((ridx_) - 1) * 32 * CPR + (ch_)]); \
        else af[buf_][((ridx_) - TN) % TM] = as_bf16x8((st_)[a_base + ((ridx_) - TN) * 32 * CPR + (ch_)]); \
    } while (0)

    // every kernel argument the epilogue needs is in registers before the loop (see the file header)
    asm volatile("" ::"s"(Cout), "s"(M), "s"(N), "s"(rope.table), "s"(rope.pos), "s"(rope.L), "s"(rope.rope_cols),
                 "s"(rope.c_panel_rows), "s"(rope.row_ssq), "s"(rope.x), "s"(rope.gain), "s"(rope.h_out), "s"(rope.ssq_out),
                 "s"(rope.tickets), "s"(rope.ssq_out_stride));
    __shared__ float s_inv[BM];
    row_scale_prologue<BM>(s_inv, m0, M, K, rope);   // (its loads are complete before the first copy is issued)

#pragma unroll
    for (int s = 0; s < P; ++s)
        if (s < nk) {
#pragma unroll
            for (int t = 0; t < LOADS; ++t) DLLM_COPY(t, s, s);
        }
    wait_stages_after<P - 1, LOADS>(min(P, nk) - 1);
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
#pragma unroll
    for (int r = 0; r < NRD; ++r) DLLM_READ(r, smem, lhalf ^ sw, 0);

    // The K loop exists twice: SKIP = false multiplies every sub-tile, with no branch between the MFMAs
    // (every workgroup but those of a ragged last row tile); SKIP = true tests each MFMA's sub-tile.
    auto k_loop = [&](auto skip_tag) __attribute__((always_inline)) {
    constexpr bool SKIP = decltype(skip_tag)::value;
    int slot = 0, cslot = P % NST;  // slot of stage kt; slot that receives stage kt + P
    int kt = 0;
#pragma unroll
    for (int phase = 0; phase < 2; ++phase) {
        // phase 0: steady state, every step also copies stage kt + P; phase 1: the last P steps
        const int kt_end = phase == 0 ? max(0, nk - P) : nk;
        for (; kt < kt_end; ++kt) {
            const int next_slot = slot + 1 == NST ? 0 : slot + 1;
            const uint4 *st = smem + slot * STAGE, *stn = smem + next_slot * STAGE;
#pragma unroll
            for (int kk = 0; kk < KS; ++kk) {
                const int cur = kk & 1, nxt = cur ^ 1;
                const bool last = kk == KS - 1;
                const uint4 *rs = last ? stn : st;
                const int ch = last ? (lhalf ^ sw) : (((kk + 1) * 2 + lhalf) ^ sw);
                if (last) {
                    // every read of this stage has returned; stage kt+1 has landed for this wave, and
                    // after the barrier for all of them; the slot of stage kt-1 was free a step ago
                    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                    if (phase == 0) wait_vmcnt<(P - 2) * LOADS + (KS - 1) * LOADS / KS>();
                    else wait_stages_after<P - 2, LOADS>(nk - 2 - kt);
                    __builtin_amdgcn_s_barrier();
                    asm volatile("" ::: "memory");
                }
                const int c0 = kk * LOADS / KS, c1 = (kk + 1) * LOADS / KS, NC = c1 - c0;
                // The substep in front of the barrier ends with a wait for every fragment read it issued, so
                // it issues them during its first MFMAs (the rest of its MFMAs then cover their latency) and
                // its copies during the later ones; the other substeps spread both evenly.
                const bool front = kEarlyReads && kk == KS - 2;
                constexpr int HALF = (NMF + 1) / 2, RQ = (NRD + HALF - 1) / HALF, REST = NMF - HALF, RDIV = REST > 0 ? REST : 1;
#pragma unroll
                for (int m = 0; m < NMF; ++m) {
                    const int r0 = front ? min(NRD, m * RQ) : m * NRD / NMF;
                    const int r1 = front ? min(NRD, (m + 1) * RQ) : (m + 1) * NRD / NMF;
#pragma unroll
                    for (int r = r0; r < r1; ++r) DLLM_READ(r, rs, ch, nxt);
                    if (phase == 0) {
                        const bool late = front && REST > 0;
                        const int q0 = late ? (m < HALF ? 0 : (m - HALF) * NC / RDIV) : m * NC / NMF;
                        const int q1 = late ? (m < HALF ? 0 : (m - HALF + 1) * NC / RDIV) : (m + 1) * NC / NMF;
#pragma unroll
                        for (int c = c0 + q0; c < c0 + q1; ++c) DLLM_COPY(c, kt + P, cslot);
                    }
                    if (!SKIP || m / TN < tm_valid)
                        acc[m / TN][m % TN] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[cur][m % TN], af[cur][m / TN],
                                                                                     acc[m / TN][m % TN], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);  // keeps the hand-made interleaving
                }
            }
            slot = next_slot;
            cslot = cslot + 1 == NST ? 0 : cslot + 1;
        }
    }
    };
    if (kSkipEmpty && tm_valid < TM) k_loop(std::true_type{});
    else k_loop(std::false_type{});
#undef DLLM_COPY
#undef DLLM_READ
    if constexpr (EPI == kEpiResidual) {
        residual_finish<TM, TN, WTM, WN>(acc, Cout, M, N, m0, n0, wm, wn, l32, lhalf, pid_n, rope);
        return;
    }
    const float *inv = rope.row_ssq ? s_inv : nullptr;   // written before the K loop's barriers
    const int n_lim = epi_paired(EPI) ? N / 2 : N;
    if constexpr (kSkipEmpty) {  // (the 256x256 tile has no register to spare for a second epilogue)
        if (m0 + BM <= M && n0 + BN_OUT <= n_lim && (n_lim & 3) == 0 && (N & 3) == 0) {
            store_tile<TM, TN, WTM, EPI, false>(acc, Cout, M, N, m0, n0, wm, wn, l32, lhalf, blockIdx.y, rope, inv);
            return;
        }
    }
    store_tile<TM, TN, WTM, EPI, true>(acc, Cout, M, N, m0, n0, wm, wn, l32, lhalf, blockIdx.y, rope, inv);
}

// ---- fallback kernel: any K % 8 == 0 -------------------------------------------
template <int BM, int BN, int WM, int WN, int EPI>
__global__ __launch_bounds__(WM * WN * 64) void gemm_reg_kernel(const uint16_t *__restrict__ A,
                                                            const uint16_t *__restrict__ W, void *__restrict__ Cout,
                                                            int M, int N, int K, int k_per_split, int num_m, int num_n,
                                                            RopeArgs rope)
{
    constexpr int kBK = 64, kChunksPerRow = 8;
    constexpr int kThreads = WM * WN * 64, RPL = kThreads / kChunksPerRow;  // rows covered by one load of all threads
    constexpr int WTM = BM / WM, WTN = BN / WN, TM = WTM / 32, TN = WTN / 32;
    constexpr int ROWS = BM + BN;
    constexpr int LOADS = ROWS / RPL;
    constexpr int A_LOADS = BM / RPL;
    static_assert(ROWS % RPL == 0 && BM % RPL == 0, "whole loads");
    constexpr int STAGE = ROWS * kChunksPerRow;
    extern __shared__ uint4 smem[];

    int pid_m, pid_n;
    tile_of(blockIdx.x, num_m, num_n, pid_m, pid_n);
    constexpr int BN_OUT = epi_paired(EPI) ? BN / 2 : BN;
    const int m0 = pid_m * BM, n0 = pid_n * BN_OUT;
    const int n_lim = epi_paired(EPI) ? N / 2 : N;  // columns or pairs of the matrix
    const int kbeg = blockIdx.y * k_per_split;
    const int kend = min(K, kbeg + k_per_split);
    const int nk = (kend - kbeg + kBK - 1) / kBK;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int wm = wave / WN, wn = wave % WN;
    const int l32 = lane & 31, lhalf = lane >> 5;

    const int ld_row = tid >> 3, ld_kc = tid & 7;  // + RPL rows per extra load
    const uint16_t *src[LOADS];
    bool ok[LOADS];
#pragma unroll
    for (int t = 0; t < LOADS; ++t) {
        const int r = ld_row + t * RPL;
        int grow;
        if (t < A_LOADS) {
            ok[t] = m0 + r < M;
            grow = m0 + r;
        } else {
            const int j = r - BM;
            ok[t] = epi_paired(EPI) ? (n0 + (j >> 5) * 16 + (j & 15) < n_lim) : (n0 + j < n_lim);
            grow = w_global_row<EPI>(j, n0, N);
        }
        src[t] = (t < A_LOADS ? A : W) + (size_t)(ok[t] ? grow : 0) * K + ld_kc * 8;
    }
    uint4 reg[LOADS];

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;
    int a_row[TM], b_row[TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) a_row[i] = (wm * WTM + i * 32 + l32) * kChunksPerRow;
#pragma unroll
    for (int j = 0; j < TN; ++j) b_row[j] = (BM + wn * WTN + j * 32 + l32) * kChunksPerRow;
    const int sw = (l32 >> 1) & 7;
    __shared__ float s_inv[BM];
    row_scale_prologue<BM>(s_inv, m0, M, K, rope);   // (read after the loop's barriers)

    for (int kt = 0; kt <= nk; ++kt) {
        // registers of step kt-1 go to LDS, step kt is fetched, step kt-1 is multiplied
        if (kt > 0) {
            uint4 *dst = smem + ((kt - 1) & 1) * STAGE;
#pragma unroll
            for (int t = 0; t < LOADS; ++t) {
                const int r = ld_row + t * RPL;
                dst[r * kChunksPerRow + (ld_kc ^ ((r >> 1) & 7))] = reg[t];
            }
        }
        if (kt < nk) {
            const int k = kbeg + kt * kBK;
            const bool kin = k + ld_kc * 8 < kend;
#pragma unroll
            for (int t = 0; t < LOADS; ++t)
                reg[t] = (ok[t] && kin) ? *reinterpret_cast<const uint4 *>(src[t] + k) : make_uint4(0, 0, 0, 0);
        }
        __syncthreads();
        if (kt == 0) continue;
        const uint4 *st = smem + ((kt - 1) & 1) * STAGE;
#pragma unroll
        for (int kk = 0; kk < kBK / 16; ++kk) {
            const int ch = (kk * 2 + lhalf) ^ sw;
            bf16x8 af[TM], bfr[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) af[i] = as_bf16x8(st[a_row[i] + ch]);
#pragma unroll
            for (int j = 0; j < TN; ++j) bfr[j] = as_bf16x8(st[b_row[j] + ch]);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af[i], acc[i][j], 0, 0, 0);
        }
    }
    if constexpr (EPI == kEpiResidual) {
        residual_finish<TM, TN, WTM, WN>(acc, Cout, M, N, m0, n0, wm, wn, l32, lhalf, pid_n, rope);
        return;
    }
    store_tile<TM, TN, WTM, EPI, true>(acc, Cout, M, N, m0, n0, wm, wn, l32, lhalf, blockIdx.y, rope,
                                       rope.row_ssq ? s_inv : nullptr);
}

// ---- host side ----------------------------------------------------------------

// Tile shapes with the modelled cost of one 64-deep K-step and of the epilogue in
// microseconds when every CU holds a workgroup (measured on MI355X with random
// operands; under that load the shader clock sits near 1.5 GHz; the three 256-row
// tiles are fitted to many-round runs at M = 4096 and 12288 as well as to M = 512:
// per round of 64 K-steps the 256x256 tile takes 115-120 us, 256x192 99-105 us,
// 256x128 66-77 us, so the largest tile is the cheapest per flop once M fills it).
struct TileCfg {
    int bm, bn, bk, nst, wn;  // wn: wave columns of the tile
    float step_us, epi_us;
};
constexpr int kNumCfg = 10;
const TileCfg kCfg[kNumCfg] = {
    {256, 256, 32, 4, 2, 1.70f, 9.0f}, {256, 192, 32, 5, 2, 1.45f, 8.0f}, {256, 128, 64, 3, 2, 0.97f, 6.0f},
    {256, 96, 64, 3, 1, 0.77f, 5.0f},  {128, 128, 64, 4, 2, 0.62f, 3.5f}, {128, 64, 64, 4, 2, 1.00f, 2.5f},
    {64, 64, 64, 8, 2, 0.30f, 1.5f},  // few rows (cached steps): a deep ring keeps 56 KB of weights in flight per workgroup
    // 32-deep stages with deep rings: with panel-major operands a 64-byte row piece is as cheap a request as a
    // 128-byte one, and the ring then looks further ahead in time
    {128, 192, 32, 7, 2, 0.72f, 5.0f}, {256, 128, 32, 6, 2, 1.00f, 6.0f}, {128, 128, 32, 8, 2, 0.66f, 3.5f},
};
constexpr int kNumCU = 256;
constexpr int kLdsPerCU = 160 * 1024;
// Weight streaming: a workgroup keeps (NST - 1) stages of its W tile in flight and a request takes about
// 2 us under load, so few or shallow workgroups cannot pull the ~4.3 TB/s the HBM delivers to this pattern
// (measured on the vocabulary projection at M = 256, where every workgroup streams a W tile of its own).
constexpr double kHbmBytesPerUs = 4.3e6, kLoadLatencyUs = 2.0;

struct Plan {
    int cfg, splits;
    bool fast;  // gemm_il_kernel
};

// Test and tuning hooks from the environment, read once (and again by gemm_reload_env): DLLM_GEMM_FALLBACK
// forces the register-staged kernel, DLLM_NO_FUSED_ROPE the separate rotary kernel, DLLM_GEMM_CFG a tile
// shape for every product, DLLM_GEMM_CFG_E<epilogue> for one epilogue, DLLM_GEMM_SPLITS a split count;
// DLLM_GEMM_ONLY_K restricts the tile and split overrides to products with that inner dimension.
constexpr int kNumEpi = 7;
struct EnvHooks {
    bool loaded = false;
    int fallback = 0, no_fused_rope = 0, cfg_all = -1, cfg_epi[kNumEpi] = {-1, -1, -1, -1, -1, -1, -1}, splits = -1, only_k = 0;
};
std::mutex g_plan_mutex;  // guards g_env and g_plans
EnvHooks g_env;
std::map<std::tuple<int, int, int, int, int>, Plan> g_plans;  // (epilogue, M, N, K, split limit) -> plan

int env_int(const char *name, int dflt)
{
    const char *s = getenv(name);
    return s ? atoi(s) : dflt;
}

void load_env_locked()
{
    g_env.fallback = env_int("DLLM_GEMM_FALLBACK", 0);
    g_env.no_fused_rope = env_int("DLLM_NO_FUSED_ROPE", 0);
    g_env.cfg_all = env_int("DLLM_GEMM_CFG", -1);
    for (int e = 0; e < kNumEpi; ++e) {
        char name[32];
        snprintf(name, sizeof name, "DLLM_GEMM_CFG_E%d", e);
        g_env.cfg_epi[e] = env_int(name, -1);
    }
    g_env.splits = env_int("DLLM_GEMM_SPLITS", -1);
    g_env.only_k = env_int("DLLM_GEMM_ONLY_K", 0);
    g_env.loaded = true;
}

EnvHooks env_hooks()
{
    std::lock_guard<std::mutex> lock(g_plan_mutex);
    if (!g_env.loaded) load_env_locked();
    return g_env;
}

// epi: a GemmEpilogue value or one of the rotary epilogues
bool cfg_allows(int c, int epi, bool fast)
{
    if (!fast && c < 2) return false;  // the register-staged kernel keeps to the smaller tiles
    // 256 accumulator registers per lane leave no room for the addresses of the fp32 epilogues (the residual
    // epilogue compiles with 360 bytes of scratch per lane), and at N = 4096 it measured no faster than the
    // 256x128 tile (B = 8, L = 1536: 162.4-162.6 ms per step either way)
    if (c == 0 && (epi == kEpiPartial || epi == kEpiResidual)) return false;
    // a wave's slice of a row is at least 64 columns wide, which bounds the partial results per row
    if (epi == kEpiRowStats && kCfg[c].bn / kCfg[c].wn < 64) return false;
    return true;
}

// Lowest modelled time: rounds of workgroups over the CUs, each round costing
// the K-steps of one tile plus its epilogue, plus the traffic of the fp32 slabs.
Plan search_plan(const EnvHooks &env, int epi, int M, int N, int K, int split_limit)
{
    const int n_out = epi == kEpiSwiglu ? N / 2 : N;
    // the asynchronous-copy kernel needs whole K-steps and 32-bit byte offsets
    const bool fast = (K % 64 == 0) && ((double)M * K * 2 < 4.0e9) && ((double)N * K * 2 < 4.0e9) && env.fallback == 0;
    const bool forced = env.only_k <= 0 || env.only_k == K;
    const int fc = !forced ? -1 : (epi >= 0 && epi < kNumEpi && env.cfg_epi[epi] >= 0) ? env.cfg_epi[epi] : env.cfg_all;
    const int fs = forced ? env.splits : -1;
    Plan best{4, 1, fast};
    double best_cost = 1e300;
    const bool splittable = epi == kEpiPartial || epi == kEpiResidual;
    const int max_splits = splittable ? (split_limit < 1 ? 1 : split_limit > kGemmMaxSplits ? kGemmMaxSplits : split_limit) : 1;
    for (int c = 0; c < kNumCfg; ++c) {
        if (!cfg_allows(c, epi, fast) || (fc >= 0 && fc < kNumCfg && cfg_allows(fc, epi, fast) && c != fc)) continue;
        // a single row of 256x256 tiles that only streams W and writes bf16 logits measured 315 us where the model
        // says 271 and the 256x128 tile takes 284 (row-major operands); with the row-statistics epilogue, panel-major
        // weights and non-temporal copies the largest tile is the fastest (228 vs 250-257 us at 256 rows) and stays in
        if (c == 0 && fc != 0 && M < 1024 && epi == kEpiBf16 && N > 16 * K) continue;
        const TileCfg &t = kCfg[c];
        const int bn_out = epi == kEpiSwiglu ? t.bn / 2 : t.bn;
        const long tiles = (long)((M + t.bm - 1) / t.bm) * ((n_out + bn_out - 1) / bn_out);
        for (int s = 1; s <= max_splits; ++s) {
            if (fs >= 1 && fs <= max_splits && s != fs) continue;
            const int kps = ((K + s - 1) / s + 63) / 64 * 64;
            if (s > 1 && (long)kps * (s - 1) >= K) continue;  // the last split would be empty
            const long wgs = tiles * s;
            const long rounds = (wgs + kNumCU - 1) / kNumCU;
            // a round that leaves CUs idle runs its workgroups faster (power and bandwidth are shared by fewer)
            const double fill = (double)wgs / (double)(rounds * kNumCU);
            // sub-tiles without rows are skipped by the kernel
            const int m_tiles = (M + t.bm - 1) / t.bm;
            const double rows_frac = (double)((M + 31) / 32 * 32) / (double)(m_tiles * t.bm);
            const double compute = (double)rounds * (double)(kps / 64) * t.step_us * (0.55 + 0.45 * fill) * rows_frac;
            const int per_cu = kLdsPerCU / (t.nst * (t.bm + t.bn) * t.bk * 2) >= 2 ? 2 : 1;
            const double in_flight = (double)(wgs < (long)kNumCU * per_cu ? wgs : (long)kNumCU * per_cu) *
                                     (double)((t.nst - 1) * t.bn * t.bk * 2);
            const double bw = in_flight / kLoadLatencyUs < kHbmBytesPerUs ? in_flight / kLoadLatencyUs : kHbmBytesPerUs;
            const long cap = (long)kNumCU * per_cu;  // a partly filled last round streams at a lower rate
            const double stream = (double)N * K * 2.0 / bw * (wgs > cap ? (double)((wgs + cap - 1) / cap * cap) / (double)wgs : 1.0);
            double cost = (compute > stream ? compute : stream) + (double)rounds * (t.epi_us + 1.5);
            if (splittable) cost += (double)s * M * N * 8.0 / 4.0e6;  // slab write + read, ~4 TB/s
            if (cost < best_cost) { best_cost = cost; best = Plan{c, s, fast}; }
        }
    }
    return best;
}

// The plan of a product is searched once per (epilogue, shape, split limit) and kept.
Plan make_plan(int epi, int M, int N, int K, int split_limit = kGemmMaxSplits)
{
    const auto key = std::make_tuple(epi, M, N, K, split_limit);
    std::lock_guard<std::mutex> lock(g_plan_mutex);
    if (!g_env.loaded) load_env_locked();
    auto it = g_plans.find(key);
    if (it != g_plans.end()) return it->second;
    const Plan p = search_plan(g_env, epi, M, N, K, split_limit);
    g_plans.emplace(key, p);
    return p;
}

// Pitches of the kernel's operand addressing for a layout (see the kernel); false if a panel-major operand
// is asked of a kernel that cannot read it or does not fit 32-bit offsets.
void set_scale(RopeArgs &r, const RowScale &sc)
{
    r.row_ssq = sc.ssq; r.ssq_parts = sc.parts; r.ssq_stride = sc.stride; r.eps = sc.eps;
}

bool set_layout(RopeArgs &r, const GemmLayout &lay, bool fast, int K)
{
    if (!fast && (lay.a_panel_rows || lay.w_panel_rows)) return false;   // (outputs are written by the shared epilogues)
    if ((double)lay.a_panel_rows * 64 * 2 >= 4.0e9 || (double)lay.w_panel_rows * 64 * 2 >= 4.0e9) return false;
    r.a_row_pitch = lay.a_panel_rows ? 64u : (uint32_t)K * 2u;
    r.a_panel_pitch = lay.a_panel_rows ? (uint32_t)lay.a_panel_rows * 64u : 64u;
    r.w_row_pitch = lay.w_panel_rows ? 64u : (uint32_t)K * 2u;
    r.w_panel_pitch = lay.w_panel_rows ? (uint32_t)lay.w_panel_rows * 64u : 64u;
    r.c_panel_rows = lay.c_panel_rows;
    return true;
}

template <int BM, int BN, int WM, int WN, int BK, int NST, int EPI>
hipError_t launch_cfg(hipStream_t stream, bool fast, const void *A, const void *W, void *C, int M, int N, int K,
                      int splits, RopeArgs rope)
{
    constexpr int BN_OUT = epi_paired(EPI) ? BN / 2 : BN;
    const int n_lim = epi_paired(EPI) ? N / 2 : N;
    const int num_m = (M + BM - 1) / BM, num_n = (n_lim + BN_OUT - 1) / BN_OUT;
    const int kps = ((K + splits - 1) / splits + 63) / 64 * 64;
    const dim3 grid(num_m * num_n, splits), block(WM * WN * 64);
    if (fast) {
        const size_t lds = (size_t)NST * (BM + BN) * BK * 2;
        auto kern = gemm_il_kernel<BM, BN, WM, WN, BK, NST, EPI>;
        // once per kernel, whichever thread comes first (initialisation of a local static is thread-safe)
        static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (attr != hipSuccess) return attr;
        hipLaunchKernelGGL(kern, grid, block, lds, stream, (const uint16_t *)A, (const uint16_t *)W, C, M, N, K, kps,
                           num_m, num_n, rope);
    } else if constexpr (BM * BN > 256 * 128) {
        return hipErrorInvalidValue;  // never planned: see cfg_allows
    } else {
        const size_t lds = (size_t)2 * (BM + BN) * 128;
        auto kern = gemm_reg_kernel<BM, BN, WM, WN, EPI>;
        static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (attr != hipSuccess) return attr;
        hipLaunchKernelGGL(kern, grid, block, lds, stream, (const uint16_t *)A, (const uint16_t *)W, C, M, N, K, kps,
                           num_m, num_n, rope);
    }
    return hipGetLastError();
}

template <int EPI>
hipError_t dispatch(hipStream_t stream, Plan p, const void *A, const void *W, void *C, int M, int N, int K,
                    const GemmLayout &lay, RopeArgs rope = RopeArgs{})
{
    if (!set_layout(rope, lay, p.fast, K)) return hipErrorInvalidValue;
    switch (p.cfg) {
    case 0:
        if constexpr (EPI != kEpiPartial && EPI != kEpiResidual)
            return launch_cfg<256, 256, 2, 2, 32, 4, EPI>(stream, p.fast, A, W, C, M, N, K, p.splits, rope);
        return hipErrorInvalidValue;  // never planned: see cfg_allows
    case 1: return launch_cfg<256, 192, 2, 2, 32, 5, EPI>(stream, p.fast, A, W, C, M, N, K, p.splits, rope);
    case 2: return launch_cfg<256, 128, 2, 2, 64, 3, EPI>(stream, p.fast, A, W, C, M, N, K, p.splits, rope);
    case 3: return launch_cfg<256, 96, 4, 1, 64, 3, EPI>(stream, p.fast, A, W, C, M, N, K, p.splits, rope);
    case 4: return launch_cfg<128, 128, 2, 2, 64, 4, EPI>(stream, p.fast, A, W, C, M, N, K, p.splits, rope);
    case 5: return launch_cfg<128, 64, 2, 2, 64, 4, EPI>(stream, p.fast, A, W, C, M, N, K, p.splits, rope);
    case 6: return launch_cfg<64, 64, 2, 2, 64, 8, EPI>(stream, p.fast, A, W, C, M, N, K, p.splits, rope);
    case 7: return launch_cfg<128, 192, 2, 2, 32, 7, EPI>(stream, p.fast, A, W, C, M, N, K, p.splits, rope);
    case 8: return launch_cfg<256, 128, 2, 2, 32, 6, EPI>(stream, p.fast, A, W, C, M, N, K, p.splits, rope);
    default: return launch_cfg<128, 128, 2, 2, 32, 8, EPI>(stream, p.fast, A, W, C, M, N, K, p.splits, rope);
    }
}

}  // namespace

int gemm_num_splits(int M, int N, int K, int split_limit) { return make_plan(kEpiPartial, M, N, K, split_limit).splits; }

GemmPlanInfo gemm_plan_info(int epi, int M, int N, int K, int split_limit)
{
    const Plan p = make_plan(epi, M, N, K, split_limit);
    const TileCfg &t = kCfg[p.cfg];
    return GemmPlanInfo{t.bm, t.bn, p.fast ? t.bk : 64, p.fast ? t.nst : 2, 4 / t.wn, t.wn, p.splits, p.fast ? 1 : 0};
}

void gemm_reload_env()
{
    std::lock_guard<std::mutex> lock(g_plan_mutex);
    load_env_locked();
    g_plans.clear();
}

bool gemm_qkv_rope_supported(int M, int d, int dh)
{
    // pairs (c, c + dh/2) in groups of 16 inside one head; the q/k boundary on a head edge; asynchronous-copy kernel
    const EnvHooks env = env_hooks();
    return (dh == 64 || dh == 128) && d % dh == 0 && d % 64 == 0 && (double)M * d * 2 < 4.0e9 &&
           (double)3 * d * d * 2 < 4.0e9 && env.fallback == 0 && env.no_fused_rope == 0;
}

hipError_t launch_gemm_qkv_rope(hipStream_t stream, const void *A, const void *W, void *C, int M, int d, int dh,
                                const float2 *table, int L, const int32_t *pos, const GemmLayout &lay, const RowScale &scale,
                                void *kv_dst, const int32_t *kv_rows)
{
    if ((kv_dst == nullptr) != (kv_rows == nullptr)) return hipErrorInvalidValue;
    RopeArgs rope{};
    rope.table = table; rope.pos = pos; rope.L = L; rope.rope_cols = 2 * d;
    rope.kv_dst = reinterpret_cast<uint16_t *>(kv_dst); rope.kv_rows = kv_rows;
    set_scale(rope, scale);
    const Plan p = make_plan(dh == 128 ? kEpiRope128 : kEpiRope64, M, 3 * d, d);
    if (dh == 128) return dispatch<kEpiRope128>(stream, p, A, W, C, M, 3 * d, d, lay, rope);
    return dispatch<kEpiRope64>(stream, p, A, W, C, M, 3 * d, d, lay, rope);
}

size_t gemm_rowstats_max_parts(int N) { return (size_t)(N + 63) / 64 + 1; }

hipError_t launch_gemm_rowstats(hipStream_t stream, const void *A, const void *W, float *stats, int M, int N, int K,
                                int mask_id, int *parts, const GemmLayout &lay, const RowScale &scale)
{
    const Plan p = make_plan(kEpiRowStats, M, N, K);
    const TileCfg &t = kCfg[p.cfg];
    *parts = (N + t.bn - 1) / t.bn * t.wn;
    if ((size_t)*parts > gemm_rowstats_max_parts(N)) return hipErrorInvalidValue;
    RopeArgs ea{};
    ea.parts = *parts;
    ea.mask_id = mask_id;
    set_scale(ea, scale);
    return dispatch<kEpiRowStats>(stream, p, A, W, stats, M, N, K, lay, ea);
}

hipError_t launch_gemm(hipStream_t stream, GemmEpilogue epi, const void *A, const void *W, void *C, int M, int N,
                       int K, int split_limit, const GemmLayout &lay, const RowScale &scale)
{
    const Plan p = make_plan(epi, M, N, K, split_limit);
    RopeArgs ea{};
    ea.L = 1;
    switch (epi) {
    case kEpiBf16: set_scale(ea, scale); return dispatch<kEpiBf16>(stream, p, A, W, C, M, N, K, lay, ea);
    case kEpiSwiglu: set_scale(ea, scale); return dispatch<kEpiSwiglu>(stream, p, A, W, C, M, N, K, lay, ea);
    default:
        if (scale.ssq) return hipErrorInvalidValue;   // slabs of partial products cannot be scaled row by row
        return dispatch<kEpiPartial>(stream, p, A, W, C, M, N, K, lay, ea);
    }
}

hipError_t launch_gemm_residual(hipStream_t stream, const void *A, const void *W, const ResidualOut &out, int M, int N,
                                int K, int split_limit, const GemmLayout &lay, int *ssq_parts)
{
    if (!out.x || !out.gain || !out.h || !out.ssq || !out.slabs || !out.tickets || (N & 3)) return hipErrorInvalidValue;
    const Plan p = make_plan(kEpiResidual, M, N, K, split_limit);
    const TileCfg &t = kCfg[p.cfg];
    const int num_m = (M + t.bm - 1) / t.bm, num_n = (N + t.bn - 1) / t.bn;
    *ssq_parts = num_n * t.wn;
    if (*ssq_parts > out.ssq_stride || (long)num_m * num_n > out.n_tickets) return hipErrorInvalidValue;
    RopeArgs ea{};
    ea.L = 1;
    ea.x = out.x; ea.gain = (const uint16_t *)out.gain; ea.h_out = (uint16_t *)out.h; ea.ssq_out = out.ssq;
    ea.tickets = out.tickets; ea.ssq_out_stride = out.ssq_stride;
    GemmLayout l2 = lay;
    l2.c_panel_rows = out.h_panel_rows;
    return dispatch<kEpiResidual>(stream, p, A, W, out.slabs, M, N, K, l2, ea);
}

int gemm_residual_max_parts(int N) { return (N + 63) / 64 * 2; }   // narrowest tile: 64 columns, two wave columns

bool gemm_async_copy_path(int epi, int M, int N, int K, int split_limit)
{
    return make_plan(epi, M, N, K, split_limit).fast;
}

namespace {
// dst[K / 32][rows][32] = src[rows][K], 16 bytes per thread; K % 32 == 0
__global__ __launch_bounds__(256) void pack_panels_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst,
                                                          size_t rows, int chunks_per_row)
{
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= rows * chunks_per_row) return;
    const size_t r = idx / chunks_per_row;
    const int c = (int)(idx - r * chunks_per_row);
    dst[((size_t)(c >> 2) * rows + r) * 4 + (c & 3)] = src[idx];
}
}  // namespace

hipError_t launch_pack_panels(hipStream_t stream, const void *src, void *dst, size_t rows, int K)
{
    if (K % 32 || rows == 0) return hipErrorInvalidValue;
    const size_t n = rows * (size_t)(K / 8);
    if ((n + 255) / 256 > 0x7fffffffull) return hipErrorInvalidValue;
    hipLaunchKernelGGL(pack_panels_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, (const uint4 *)src,
                       (uint4 *)dst, rows, K / 8);
    return hipGetLastError();
}

}  // namespace dllm
