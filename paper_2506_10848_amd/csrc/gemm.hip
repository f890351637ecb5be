// bf16 MFMA GEMM for gfx950:  C = A[M][K] * W[N][K]^T, fp32 accumulation.
//
// Both operands are K-contiguous, which is what the 32x32x16 bf16 MFMA wants: a
// lane feeds 8 consecutive K values of one row (A) or one column (W).  A
// workgroup of 4 or 8 waves owns a BM x BN tile (8 waves, two per SIMD, keep the
// LDS pipe busier: a single wave per SIMD cannot keep enough fragment reads in
// flight) and walks K in steps of 64 through a
// multi-stage LDS ring.
//
// Main kernel (gemm_dl_kernel, K % 64 == 0):
//   * global -> LDS copies are asynchronous (global_load_lds_dwordx4, 1 KB per
//     wave instruction, no VGPR staging) and run NST-1 K-steps ahead of the math;
//     the only per-step synchronisation is one s_waitcnt vmcnt + one s_barrier.
//   * LDS rows are 128 bytes; 16-byte chunks are XOR-swizzled with (row >> 1) & 7.
//     The LDS has 64 banks and serves 16 lanes x 16 bytes per cycle, i.e. two rows
//     per cycle, so this keeps the fragment reads of 16 consecutive rows on 64
//     distinct banks.  The swizzle is applied by choosing which global chunk each
//     lane copies, because the LDS side of the copy is fixed (lane * 16 bytes).
//   * fragments for K-substep kk+1 are requested before the MFMAs of substep kk
//     (scheduling barriers keep the compiler from sinking the reads again).
//   * MFMAs are issued as (W fragment) x (A fragment): the accumulators then hold
//     the transposed tile, four consecutive output columns per lane, and the
//     epilogue stores 8 (bf16) or 16 (fp32) bytes per lane.
// Fallback kernel (gemm_reg_kernel): any K % 8 == 0, register-staged loads with
// zero fill, two LDS stages.
//
// Epilogues: bf16 store; SwiGLU (a tile carries the gate and the up columns of
// the same features, so silu(gate) * up is formed in registers); fp32 slabs for
// split-K, which the next residual-add + RMSNorm kernel sums.
//
// Workgroup ids are mapped so that the tiles sharing a weight column block run on
// the same XCD (ids congruent mod 8 share an L2).
#include <stdlib.h>

#include "internal.h"

namespace dllm {

namespace {

constexpr int kBK = 64;           // K elements per LDS stage
constexpr int kChunksPerRow = 8;  // 16-byte chunks in a 64-element bf16 row

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
__device__ __forceinline__ void async_load16(const char *base_uniform, uint32_t voffset, uint32_t lds_addr_uniform)
{
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

// tile of this workgroup; tiles that share W rows get ids congruent mod 8
__device__ __forceinline__ void tile_of(int pid, int num_m, int num_n, int &pid_m, int &pid_n)
{
    const int n8 = num_n & ~7, head = num_m * n8;
    if (pid < head) {
        const int xcd = pid & 7, j = pid >> 3;
        pid_m = j % num_m;
        pid_n = (j / num_m) * 8 + xcd;
    } else {
        const int r = pid - head;
        pid_m = r % num_m;
        pid_n = n8 + r / num_m;
    }
}

// Rotary embedding fused into the QKV projection's epilogue (kEpiRope): output
// columns below rope_cols (the q and k thirds) are rotated in fp32 before the
// bf16 rounding; pos = row % L, table[pos][j] = (cos, sin) of pos * theta^(-2j/dh).
struct RopeArgs {
    const float2 *table;
    int L, dh, rope_cols;
};
constexpr int kEpiRope64 = 3, kEpiRope128 = 4;  // head_dim is a compile-time constant of the epilogue

// Accumulators hold the transposed 32x32 tiles: element e of lane l is output
// row l % 32, column 8*(e/4) + 4*(l/32) + e%4.
template <int TM, int TN, int WTM, int WTN, int EPI>
__device__ __forceinline__ void store_tile(floatx16 (&acc)[TM][TN], void *Cout, int M, int N, int n_out, int m0, int n0,
                                           int wm, int wn, int l32, int lhalf, int split, const RopeArgs &rope)
{
    constexpr int HALF_TN = TN / 2 > 0 ? TN / 2 : 1;
    if (EPI == kEpiRope64 || EPI == kEpiRope128) {
        // the wave holds whole heads: columns c and c + DH/2 of a head sit in sub-tiles j and
        // j + PJ, same lane, same element
        constexpr int DH = EPI == kEpiRope128 ? 128 : 64, PJ = DH / 64;
        if (n0 + wn * WTN < rope.rope_cols) {
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const int row = m0 + wm * WTM + i * 32 + l32;
                const float2 *trow = rope.table + (size_t)(row % rope.L) * (DH / 2) + 4 * lhalf;
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    if ((j / PJ) & 1) continue;  // second half of a head: handled with its partner
                    constexpr int TNm = TN;      // (keeps the partner index inside the array for every instantiation)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        // four consecutive (cos, sin) pairs: 32 bytes
                        const float4 *tp = reinterpret_cast<const float4 *>(trow + ((j * 32) % DH) + 8 * q);
                        const float4 t01 = tp[0], t23 = tp[1];
                        const float cs[4] = {t01.x, t01.z, t23.x, t23.z}, sn[4] = {t01.y, t01.w, t23.y, t23.w};
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float a = acc[i][j][4 * q + e], b = acc[i][(j + PJ) % TNm][4 * q + e];
                            acc[i][j][4 * q + e] = a * cs[e] - b * sn[e];
                            acc[i][(j + PJ) % TNm][4 * q + e] = a * sn[e] + b * cs[e];
                        }
                    }
                }
            }
        }
    }
    if (EPI == kEpiBf16 || EPI == kEpiRope64 || EPI == kEpiRope128) {
        uint16_t *C = reinterpret_cast<uint16_t *>(Cout);
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int row = m0 + wm * WTM + i * 32 + l32;
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int col = n0 + wn * WTN + j * 32 + 8 * q + 4 * lhalf;
                    if (row >= M || col >= N) continue;
                    uint16_t *p = C + (size_t)row * N + col;
                    if (col + 3 < N && (N & 3) == 0) {
                        uint2 w;
                        w.x = pack_bf16x2(acc[i][j][4 * q], acc[i][j][4 * q + 1]);
                        w.y = pack_bf16x2(acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
                        *reinterpret_cast<uint2 *>(p) = w;
                    } else {
                        for (int e = 0; e < 4 && col + e < N; ++e) p[e] = float_to_bf16_bits(acc[i][j][4 * q + e]);
                    }
                }
        }
    } else if (EPI == kEpiSwiglu) {
        uint16_t *C = reinterpret_cast<uint16_t *>(Cout);
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int row = m0 + wm * WTM + i * 32 + l32;
#pragma unroll
            for (int j = 0; j < HALF_TN; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int col = n0 + wn * (WTN / 2) + j * 32 + 8 * q + 4 * lhalf;
                    float y[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float g = acc[i][j][4 * q + e], u = acc[i][j + HALF_TN][4 * q + e];
                        y[e] = g / (1.0f + __expf(-g)) * u;
                    }
                    if (row >= M || col >= n_out) continue;
                    uint16_t *p = C + (size_t)row * n_out + col;
                    if (col + 3 < n_out && (n_out & 3) == 0) {
                        uint2 w;
                        w.x = pack_bf16x2(y[0], y[1]);
                        w.y = pack_bf16x2(y[2], y[3]);
                        *reinterpret_cast<uint2 *>(p) = w;
                    } else {
                        for (int e = 0; e < 4 && col + e < n_out; ++e) p[e] = float_to_bf16_bits(y[e]);
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
                    const int col = n0 + wn * WTN + j * 32 + 8 * q + 4 * lhalf;
                    if (row >= M || col >= N) continue;
                    float *p = C + (size_t)row * N + col;
                    if (col + 3 < N && (N & 3) == 0) {
                        *reinterpret_cast<float4 *>(p) = make_float4(acc[i][j][4 * q], acc[i][j][4 * q + 1],
                                                                     acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
                    } else {
                        for (int e = 0; e < 4 && col + e < N; ++e) p[e] = acc[i][j][4 * q + e];
                    }
                }
        }
    }
}

// LDS row (in 16-byte chunks) of the W fragment j of wave column wn.  For the
// SwiGLU epilogue the stage holds [gate rows | up rows] and a wave pairs the
// same features from both halves.
template <int BM, int BN, int WTN, int TN, int EPI>
__device__ __forceinline__ int w_frag_row(int j, int wn, int l32)
{
    if (EPI == kEpiSwiglu) {
        constexpr int HALF_TN = TN / 2 > 0 ? TN / 2 : 1;
        return BM + (j / HALF_TN) * (BN / 2) + wn * (WTN / 2) + (j % HALF_TN) * 32 + l32;
    }
    return BM + wn * WTN + j * 32 + l32;
}

// ---- main kernel: K % 64 == 0, k_per_split % 64 == 0 --------------------------
template <int BM, int BN, int WM, int WN, int NST, int EPI>
__global__ __launch_bounds__(WM * WN * 64) void gemm_dl_kernel(const uint16_t *__restrict__ A,
                                                           const uint16_t *__restrict__ W, void *__restrict__ Cout,
                                                           int M, int N, int K, int k_per_split, int num_m, int num_n,
                                                           RopeArgs rope)
{
    constexpr int NW = WM * WN;
    static_assert(NW == 4 || NW == 8, "4 or 8 waves per workgroup");
    constexpr int WTM = BM / WM, WTN = BN / WN, TM = WTM / 32, TN = WTN / 32;
    static_assert(TM >= 1 && TN >= 1 && WTM % 32 == 0 && WTN % 32 == 0, "wave tile is made of 32x32 MFMA tiles");
    static_assert(EPI != kEpiSwiglu || TN % 2 == 0, "SwiGLU pairs gate/up sub-tiles");
    static_assert(NST >= 2 && NST <= 4, "stage count");
    constexpr int ROWS = BM + BN;             // rows of one stage: the A tile, then the W tile
    constexpr int LOADS = ROWS / (8 * NW);    // 1 KB copies per wave per stage
    constexpr int A_LOADS = BM / (8 * NW);
    static_assert(ROWS % (8 * NW) == 0 && BM % (8 * NW) == 0, "whole 8-row groups per wave");
    constexpr int STAGE = ROWS * kChunksPerRow;  // uint4 per stage
    extern __shared__ uint4 smem[];

    int pid_m, pid_n;
    tile_of(blockIdx.x, num_m, num_n, pid_m, pid_n);
    constexpr int BN_OUT = (EPI == kEpiSwiglu) ? BN / 2 : BN;
    const int m0 = pid_m * BM, n0 = pid_n * BN_OUT;
    const int n_out = (EPI == kEpiSwiglu) ? N / 2 : N;
    const int kbeg = blockIdx.y * k_per_split;
    const int kend = min(K, kbeg + k_per_split);
    const int nk = (kend - kbeg) / kBK;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int wm = wave / WN, wn = wave % WN;
    const int l32 = lane & 31, lhalf = lane >> 5;

    // wave w copies the 8-row groups w, w+NW, ...; lane l lands on row l/8, slot l%8
    // of its group and therefore fetches the chunk that the swizzle puts there
    const int lrow = lane >> 3;
    const int kc = (lane & 7) ^ (((wave & 1) << 2) | (lrow >> 1));
    uint32_t goff[LOADS];  // byte offsets into A (first A_LOADS) or W; rows past the edge are clamped
#pragma unroll
    for (int t = 0; t < LOADS; ++t) {
        const int r = 8 * (wave + NW * t) + lrow;
        int grow;
        if (t < A_LOADS) {
            grow = min(m0 + r, M - 1);
        } else if (EPI == kEpiSwiglu) {
            const int j = r - BM, half = j / (BN / 2), jj = j % (BN / 2);
            grow = half * n_out + min(n0 + jj, n_out - 1);
        } else {
            grow = min(n0 + r - BM, N - 1);
        }
        goff[t] = (uint32_t)grow * (uint32_t)K * 2u + kc * 16;
    }
    const char *Ab = reinterpret_cast<const char *>(A) + (size_t)kbeg * 2;
    const char *Wb = reinterpret_cast<const char *>(W) + (size_t)kbeg * 2;
#define DLLM_ISSUE_STAGE(kt_, stage_)                                                        \
    do {                                                                                     \
        const char *pa_ = Ab + (size_t)(kt_) * (kBK * 2), *pw_ = Wb + (size_t)(kt_) * (kBK * 2); \
        const uint32_t dst_ = lds_addr_of(smem + (stage_) * STAGE + wave * 64);              \
        _Pragma("unroll") for (int t = 0; t < LOADS; ++t)                                    \
            async_load16(t < A_LOADS ? pa_ : pw_, goff[t], dst_ + t * (NW * 1024));                 \
    } while (0)

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
    for (int j = 0; j < TN; ++j) b_row[j] = w_frag_row<BM, BN, WTN, TN, EPI>(j, wn, l32) * kChunksPerRow;
    const int sw = (l32 >> 1) & 7;

#pragma unroll
    for (int s = 0; s < NST - 1; ++s)
        if (s < nk) DLLM_ISSUE_STAGE(s, s);

    for (int kt = 0; kt < nk; ++kt) {
        // step kt has landed once only the copies issued after it are outstanding
        const int ahead = min(NST - 2, nk - 1 - kt);
        if (NST >= 4 && ahead >= 2) wait_vmcnt<2 * LOADS>();
        else if (NST >= 3 && ahead >= 1) wait_vmcnt<LOADS>();
        else wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();  // also: every wave is done reading the stage refilled below
        asm volatile("" ::: "memory");
        if (kt + NST - 1 < nk) DLLM_ISSUE_STAGE(kt + NST - 1, (kt + NST - 1) % NST);
        const uint4 *st = smem + (kt % NST) * STAGE;
        bf16x8 af[2][TM], bfr[2][TN];
#pragma unroll
        for (int i = 0; i < TM; ++i) af[0][i] = as_bf16x8(st[a_row[i] + (lhalf ^ sw)]);
#pragma unroll
        for (int j = 0; j < TN; ++j) bfr[0][j] = as_bf16x8(st[b_row[j] + (lhalf ^ sw)]);
#pragma unroll
        for (int kk = 0; kk < kBK / 16; ++kk) {
            const int cur = kk & 1, nxt = cur ^ 1;
            if (kk + 1 < kBK / 16) {
                const int ch = ((kk + 1) * 2 + lhalf) ^ sw;
#pragma unroll
                for (int i = 0; i < TM; ++i) af[nxt][i] = as_bf16x8(st[a_row[i] + ch]);
#pragma unroll
                for (int j = 0; j < TN; ++j) bfr[nxt][j] = as_bf16x8(st[b_row[j] + ch]);
            }
            __builtin_amdgcn_sched_barrier(0);  // next fragments are requested before this substep's MFMAs
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[cur][j], af[cur][i], acc[i][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
#undef DLLM_ISSUE_STAGE
    store_tile<TM, TN, WTM, WTN, EPI>(acc, Cout, M, N, n_out, m0, n0, wm, wn, l32, lhalf, blockIdx.y, rope);
}

// ---- fallback kernel: any K % 8 == 0 -------------------------------------------
template <int BM, int BN, int WM, int WN, int EPI>
__global__ __launch_bounds__(WM * WN * 64) void gemm_reg_kernel(const uint16_t *__restrict__ A,
                                                            const uint16_t *__restrict__ W, void *__restrict__ Cout,
                                                            int M, int N, int K, int k_per_split, int num_m, int num_n,
                                                            RopeArgs rope)
{
    constexpr int kThreads = WM * WN * 64, RPL = kThreads / kChunksPerRow;  // rows covered by one load of all threads
    constexpr int WTM = BM / WM, WTN = BN / WN, TM = WTM / 32, TN = WTN / 32;
    static_assert(EPI != kEpiSwiglu || (TN % 2 == 0), "SwiGLU pairs gate/up sub-tiles");
    constexpr int ROWS = BM + BN;
    constexpr int LOADS = ROWS / RPL;
    constexpr int A_LOADS = BM / RPL;
    static_assert(ROWS % RPL == 0 && BM % RPL == 0, "whole loads");
    constexpr int STAGE = ROWS * kChunksPerRow;
    extern __shared__ uint4 smem[];

    int pid_m, pid_n;
    tile_of(blockIdx.x, num_m, num_n, pid_m, pid_n);
    constexpr int BN_OUT = (EPI == kEpiSwiglu) ? BN / 2 : BN;
    const int m0 = pid_m * BM, n0 = pid_n * BN_OUT;
    const int n_out = (EPI == kEpiSwiglu) ? N / 2 : N;
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
        } else if (EPI == kEpiSwiglu) {
            const int j = r - BM, half = j / (BN / 2), jj = j % (BN / 2);
            ok[t] = n0 + jj < n_out;
            grow = half * n_out + n0 + jj;
        } else {
            ok[t] = n0 + r - BM < N;
            grow = n0 + r - BM;
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
    for (int j = 0; j < TN; ++j) b_row[j] = w_frag_row<BM, BN, WTN, TN, EPI>(j, wn, l32) * kChunksPerRow;
    const int sw = (l32 >> 1) & 7;

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
    store_tile<TM, TN, WTM, WTN, EPI>(acc, Cout, M, N, n_out, m0, n0, wm, wn, l32, lhalf, blockIdx.y, rope);
}

// ---- host side ----------------------------------------------------------------

// Tile shapes with the cost of one K-step and of the epilogue in shader clocks,
// measured on MI355X at M = 512 (copy and math of a step overlap only partly:
// the LDS port is shared by the asynchronous copies and the fragment reads).
struct TileCfg {
    int bm, bn, nst, waves;
    float step_clk, epi_clk;
};
constexpr int kNumCfg = 7;
const TileCfg kCfg[kNumCfg] = {
    {256, 256, 2, 8, 3180.f, 24000.f}, {256, 192, 2, 8, 2670.f, 18000.f}, {256, 128, 3, 8, 1730.f, 11800.f},
    {256, 128, 3, 8, 1880.f, 11800.f}, {256, 96, 3, 4, 1950.f, 8900.f},   {128, 128, 3, 8, 1175.f, 5800.f},
    {128, 64, 4, 4, 800.f, 3000.f},
};
constexpr int kNumCU = 256;
constexpr int kLdsPerCU = 160 * 1024;

struct Plan {
    int cfg, splits;
    bool fast;  // gemm_dl_kernel
};

int env_int(const char *name, int dflt)
{
    const char *s = getenv(name);
    return s ? atoi(s) : dflt;
}

bool cfg_allows(int c, GemmEpilogue epi, bool fast)
{
    if (epi == kEpiSwiglu && c == 4) return false;   // 256x96 as 4x1 waves: odd number of sub-tiles per wave
    if (epi == kEpiPartial && c == 0) return false;  // 256x256 fp32 epilogue runs out of registers
    if (!fast && c < 2) return false;                // the register-staged kernel keeps to the smaller tiles
    if (epi != kEpiPartial && c == 3) return false;  // 256x128 as 8x1 waves only pays off for the split-K shapes
    return true;
}

// Lowest modelled time: rounds of workgroups over the CUs, each round costing
// the K-steps of one tile plus its epilogue, plus the traffic of the fp32 slabs.
Plan make_plan(GemmEpilogue epi, int M, int N, int K)
{
    const int n_out = epi == kEpiSwiglu ? N / 2 : N;
    // the asynchronous-copy kernel needs whole K-steps and 32-bit byte offsets
    const bool fast = (K % kBK == 0) && ((double)M * K * 2 < 4.0e9) && ((double)N * K * 2 < 4.0e9) &&
                      env_int("DLLM_GEMM_FALLBACK", 0) == 0;
    const int fc = env_int("DLLM_GEMM_CFG", -1), fs = env_int("DLLM_GEMM_SPLITS", -1);
    Plan best{5, 1, fast};
    double best_cost = 1e300;
    const int max_splits = epi == kEpiPartial ? 8 : 1;
    for (int c = 0; c < kNumCfg; ++c) {
        if (!cfg_allows(c, epi, fast) || (fc >= 0 && fc < kNumCfg && cfg_allows(fc, epi, fast) && c != fc)) continue;
        const TileCfg &t = kCfg[c];
        const int bn_out = epi == kEpiSwiglu ? t.bn / 2 : t.bn;
        const long tiles = (long)((M + t.bm - 1) / t.bm) * ((n_out + bn_out - 1) / bn_out);
        const int per_cu = kLdsPerCU / ((fast ? t.nst : 2) * (t.bm + t.bn) * 128) >= 2 ? 2 : 1;
        for (int s = 1; s <= max_splits; ++s) {
            if (fs >= 1 && fs <= max_splits && s != fs) continue;
            const int kps = ((K + s - 1) / s + kBK - 1) / kBK * kBK;
            if (s > 1 && (long)kps * (s - 1) >= K) continue;   // the last split would be empty
            const long wgs = tiles * s;
            const long rounds = (wgs + (long)kNumCU * per_cu - 1) / ((long)kNumCU * per_cu);
            double cost = (double)rounds * per_cu * ((double)(kps / kBK) * t.step_clk + t.epi_clk + 2500.0);
            if (epi == kEpiPartial) cost += (double)s * M * N * 8.0 / (4000.0 / 2.4);  // slab write + read, ~4 TB/s
            if (cost < best_cost) { best_cost = cost; best = Plan{c, s, fast}; }
        }
    }
    return best;
}

template <int BM, int BN, int WM, int WN, int NST, int EPI>
hipError_t launch_cfg(hipStream_t stream, bool fast, const void *A, const void *W, void *C, int M, int N, int K,
                      int splits, RopeArgs rope = RopeArgs{nullptr, 1, 64, 0})
{
    constexpr int BN_OUT = EPI == kEpiSwiglu ? BN / 2 : BN;
    const int n_out = EPI == kEpiSwiglu ? N / 2 : N;
    const int num_m = (M + BM - 1) / BM, num_n = (n_out + BN_OUT - 1) / BN_OUT;
    const int kps = ((K + splits - 1) / splits + kBK - 1) / kBK * kBK;
    const dim3 grid(num_m * num_n, splits), block(WM * WN * 64);
    if (fast) {
        const size_t lds = (size_t)NST * (BM + BN) * kChunksPerRow * sizeof(uint4);
        auto kern = gemm_dl_kernel<BM, BN, WM, WN, NST, EPI>;
        static bool attr_done = false;
        if (!attr_done) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
            attr_done = true;
        }
        hipLaunchKernelGGL(kern, grid, block, lds, stream, (const uint16_t *)A, (const uint16_t *)W, C, M, N, K, kps,
                           num_m, num_n, rope);
    } else {
        const size_t lds = (size_t)2 * (BM + BN) * kChunksPerRow * sizeof(uint4);
        auto kern = gemm_reg_kernel<BM, BN, WM, WN, EPI>;
        static bool attr_done = false;
        if (!attr_done) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
            attr_done = true;
        }
        hipLaunchKernelGGL(kern, grid, block, lds, stream, (const uint16_t *)A, (const uint16_t *)W, C, M, N, K, kps,
                           num_m, num_n, rope);
    }
    return hipGetLastError();
}

template <int EPI>
hipError_t dispatch(hipStream_t stream, Plan p, const void *A, const void *W, void *C, int M, int N, int K)
{
    switch (p.cfg) {
    case 0: return launch_cfg<256, 256, 4, 2, 2, EPI>(stream, p.fast, A, W, C, M, N, K, p.splits);
    case 1: return launch_cfg<256, 192, 8, 1, 2, EPI>(stream, p.fast, A, W, C, M, N, K, p.splits);
    case 2: return launch_cfg<256, 128, 4, 2, 3, EPI>(stream, p.fast, A, W, C, M, N, K, p.splits);
    case 3: return launch_cfg<256, 128, 8, 1, 3, EPI>(stream, p.fast, A, W, C, M, N, K, p.splits);
    case 4:
        if constexpr (EPI != kEpiSwiglu) return launch_cfg<256, 96, 4, 1, 3, EPI>(stream, p.fast, A, W, C, M, N, K, p.splits);
        return hipErrorInvalidValue;
    case 5: return launch_cfg<128, 128, 4, 2, 3, EPI>(stream, p.fast, A, W, C, M, N, K, p.splits);
    default: return launch_cfg<128, 64, 4, 1, 4, EPI>(stream, p.fast, A, W, C, M, N, K, p.splits);
    }
}

}  // namespace

int gemm_num_splits(int M, int N, int K) { return make_plan(kEpiPartial, M, N, K).splits; }

bool gemm_qkv_rope_supported(int M, int d, int dh)
{
    // whole heads per 128-column tile, q/k boundary on a tile edge, asynchronous-copy kernel
    return (dh == 64 || dh == 128) && d % 128 == 0 && d % kBK == 0 && (double)M * d * 2 < 4.0e9 &&
           (double)3 * d * d * 2 < 4.0e9 && env_int("DLLM_GEMM_FALLBACK", 0) == 0 && env_int("DLLM_NO_FUSED_ROPE", 0) == 0;
}

hipError_t launch_gemm_qkv_rope(hipStream_t stream, const void *A, const void *W, void *C, int M, int d, int dh,
                                const float2 *table, int L)
{
    // 256x128 tile as 8x1 waves: a wave owns 32 rows x 128 columns = whole heads
    const RopeArgs rope{table, L, dh, 2 * d};
    if (dh == 128) return launch_cfg<256, 128, 8, 1, 3, kEpiRope128>(stream, true, A, W, C, M, 3 * d, d, 1, rope);
    return launch_cfg<256, 128, 8, 1, 3, kEpiRope64>(stream, true, A, W, C, M, 3 * d, d, 1, rope);
}

hipError_t launch_gemm(hipStream_t stream, GemmEpilogue epi, const void *A, const void *W, void *C, int M, int N,
                       int K)
{
    const Plan p = make_plan(epi, M, N, K);
    switch (epi) {
    case kEpiBf16: return dispatch<kEpiBf16>(stream, p, A, W, C, M, N, K);
    case kEpiSwiglu: return dispatch<kEpiSwiglu>(stream, p, A, W, C, M, N, K);
    default: return dispatch<kEpiPartial>(stream, p, A, W, C, M, N, K);
    }
}

}  // namespace dllm
