// bf16 MFMA GEMM for gfx950:  C = A[M][K] * W[N][K]^T, fp32 accumulation.
//
// Both operands are K-contiguous, which is exactly what the 32x32x16 bf16 MFMA
// wants: a lane feeds 8 consecutive K values of one row (A) or one column (W).
// A workgroup of 4 waves owns a BM x BN tile; K is walked in steps of 64
// through double-buffered LDS.  Each 128-byte LDS row is XOR-swizzled in units
// of 16 bytes (chunk ^= row & 7) so that the 16-byte fragment reads of 8
// consecutive rows touch all 32 banks once.  Global loads for the next K step
// are issued before the MFMAs of the current one and land in LDS afterwards.
//
// Epilogues: bf16 store; SwiGLU (the tile holds the gate and the up columns of
// the same features, so silu(gate) * up is formed in registers); fp32 slabs for
// split-K, which the next residual-add + RMSNorm kernel sums.
//
// Workgroup ids are mapped to tiles so that the workgroups sharing a weight
// column block run on the same XCD (ids congruent mod 8 share an L2).
#include <stdlib.h>

#include "internal.h"

namespace dllm {

namespace {

constexpr int kThreads = 256;
constexpr int kBK = 64;             // K elements per LDS stage
constexpr int kChunksPerRow = 8;    // 16-byte chunks in a 64-element bf16 row

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v)
{
    union { uint4 u; bf16x8 b; } c;
    c.u = v;
    return c.b;
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int EPI>
__global__ __launch_bounds__(kThreads) void gemm_kernel(const uint16_t *__restrict__ A,
                                                        const uint16_t *__restrict__ W, void *__restrict__ Cout,
                                                        int M, int N, int K, int k_per_split, int num_m, int num_n)
{
    static_assert(WAVES_M * WAVES_N == 4, "4 waves per workgroup");
    constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;  // wave tile
    constexpr int TM = WTM / 32, TN = WTN / 32;            // 32x32 MFMA tiles per wave
    static_assert(TM >= 1 && TN >= 1, "wave tile too small");
    static_assert(EPI != kEpiSwiglu || (TN % 2 == 0), "SwiGLU pairs gate/up sub-tiles");
    constexpr int A_LOADS = BM * kChunksPerRow / kThreads;
    constexpr int B_LOADS = BN * kChunksPerRow / kThreads;
    constexpr int STAGE = (BM + BN) * kChunksPerRow;  // uint4 per stage

    extern __shared__ uint4 smem[];

    // ---- which tile -------------------------------------------------------
    int pid = blockIdx.x;
    int pid_m, pid_n;
    if ((num_n & 7) == 0) {
        const int xcd = pid & 7, j = pid >> 3;
        pid_m = j % num_m;
        pid_n = (j / num_m) * 8 + xcd;
    } else {
        pid_m = pid % num_m;
        pid_n = pid / num_m;
    }
    const int m0 = pid_m * BM;
    // output features per tile column and the W rows behind the LDS B rows
    constexpr int BN_OUT = (EPI == kEpiSwiglu) ? BN / 2 : BN;
    const int n0 = pid_n * BN_OUT;
    const int n_out = (EPI == kEpiSwiglu) ? N / 2 : N;

    const int kbeg = blockIdx.y * k_per_split;
    const int kend = min(K, kbeg + k_per_split);
    const int nk = (kend - kbeg + kBK - 1) / kBK;

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    const int l32 = lane & 31, lhalf = lane >> 5;

    // ---- global -> register staging ---------------------------------------
    const int ld_row = tid >> 3, ld_kc = tid & 7;  // + t * 32 rows per extra load
    const uint16_t *a_ptr[A_LOADS];
    bool a_ok[A_LOADS];
#pragma unroll
    for (int t = 0; t < A_LOADS; ++t) {
        const int grow = m0 + ld_row + t * 32;
        a_ok[t] = grow < M;
        a_ptr[t] = A + (size_t)(a_ok[t] ? grow : 0) * K + ld_kc * 8;
    }
    const uint16_t *b_ptr[B_LOADS];
    bool b_ok[B_LOADS];
#pragma unroll
    for (int t = 0; t < B_LOADS; ++t) {
        const int j = ld_row + t * 32;  // LDS B row
        int wrow;
        bool ok;
        if (EPI == kEpiSwiglu) {
            const int half = j / (BN / 2), jj = j % (BN / 2);
            ok = n0 + jj < n_out;
            wrow = half * n_out + n0 + jj;
        } else {
            ok = n0 + j < N;
            wrow = n0 + j;
        }
        b_ok[t] = ok;
        b_ptr[t] = W + (size_t)(ok ? wrow : 0) * K + ld_kc * 8;
    }

    uint4 a_reg[A_LOADS], b_reg[B_LOADS];
    auto load_global = [&](int kt) {
        const int k = kbeg + kt * kBK;
        const bool kin = k + ld_kc * 8 < kend;
#pragma unroll
        for (int t = 0; t < A_LOADS; ++t)
            a_reg[t] = (a_ok[t] && kin) ? *reinterpret_cast<const uint4 *>(a_ptr[t] + k) : make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int t = 0; t < B_LOADS; ++t)
            b_reg[t] = (b_ok[t] && kin) ? *reinterpret_cast<const uint4 *>(b_ptr[t] + k) : make_uint4(0, 0, 0, 0);
    };
    auto store_lds = [&](int stage) {
        uint4 *as = smem + stage * STAGE;
        uint4 *bs = as + BM * kChunksPerRow;
#pragma unroll
        for (int t = 0; t < A_LOADS; ++t) {
            const int row = ld_row + t * 32;
            as[row * kChunksPerRow + (ld_kc ^ (row & 7))] = a_reg[t];
        }
#pragma unroll
        for (int t = 0; t < B_LOADS; ++t) {
            const int row = ld_row + t * 32;
            bs[row * kChunksPerRow + (ld_kc ^ (row & 7))] = b_reg[t];
        }
    };

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    // LDS rows of this wave's fragments
    int a_row[TM], b_row[TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) a_row[i] = wm * WTM + i * 32 + l32;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        if (EPI == kEpiSwiglu) {
            constexpr int HALF_TN = TN / 2 > 0 ? TN / 2 : 1;
            b_row[j] = (j / HALF_TN) * (BN / 2) + wn * (WTN / 2) + (j % HALF_TN) * 32 + l32;
        } else {
            b_row[j] = wn * WTN + j * 32 + l32;
        }
    }
    const int sw = l32 & 7;

    if (nk > 0) {
        load_global(0);
        store_lds(0);
    }
    __syncthreads();

    for (int kt = 0; kt < nk; ++kt) {
        const bool more = kt + 1 < nk;
        if (more) load_global(kt + 1);
        const uint4 *as = smem + (kt & 1) * STAGE;
        const uint4 *bs = as + BM * kChunksPerRow;
#pragma unroll
        for (int kk = 0; kk < kBK / 16; ++kk) {
            const int ch = (kk * 2 + lhalf) ^ sw;
            bf16x8 af[TM], bfr[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) af[i] = as_bf16x8(as[a_row[i] * kChunksPerRow + ch]);
#pragma unroll
            for (int j = 0; j < TN; ++j) bfr[j] = as_bf16x8(bs[b_row[j] * kChunksPerRow + ch]);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
        }
        if (more) store_lds((kt + 1) & 1);
        __syncthreads();
    }

    // ---- epilogue -----------------------------------------------------------
    // accumulator element e of lane l sits at row 8*(e/4) + 4*(l/32) + e%4, column l%32
    if (EPI == kEpiBf16) {
        uint16_t *C = reinterpret_cast<uint16_t *>(Cout);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int col = n0 + wn * WTN + j * 32 + l32;
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int row = m0 + wm * WTM + i * 32 + 8 * (e / 4) + 4 * lhalf + (e % 4);
                    if (row < M && col < N) C[(size_t)row * N + col] = float_to_bf16_bits(acc[i][j][e]);
                }
            }
    } else if (EPI == kEpiSwiglu) {
        uint16_t *C = reinterpret_cast<uint16_t *>(Cout);
        constexpr int HALF_TN = TN / 2 > 0 ? TN / 2 : 1;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < HALF_TN; ++j) {
                const int col = n0 + wn * (WTN / 2) + j * 32 + l32;
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int row = m0 + wm * WTM + i * 32 + 8 * (e / 4) + 4 * lhalf + (e % 4);
                    const float g = acc[i][j][e], u = acc[i][j + HALF_TN][e];
                    const float y = g / (1.0f + __expf(-g)) * u;
                    if (row < M && col < n_out) C[(size_t)row * n_out + col] = float_to_bf16_bits(y);
                }
            }
    } else {
        float *C = reinterpret_cast<float *>(Cout) + (size_t)blockIdx.y * M * N;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int col = n0 + wn * WTN + j * 32 + l32;
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int row = m0 + wm * WTM + i * 32 + 8 * (e / 4) + 4 * lhalf + (e % 4);
                    if (row < M && col < N) C[(size_t)row * N + col] = acc[i][j][e];
                }
            }
    }
}

// ---- host side ----------------------------------------------------------------

struct TileCfg {
    int bm, bn;
    float eff;  // relative MFMA efficiency of the tile shape (bigger tiles reuse more)
};
constexpr int kNumCfg = 4;
const TileCfg kCfg[kNumCfg] = {{256, 256, 1.00f}, {256, 128, 0.85f}, {128, 128, 0.65f}, {128, 64, 0.40f}};
constexpr int kNumCU = 256;

struct Plan {
    int cfg, splits;
};

int env_int(const char *name, int dflt)
{
    const char *s = getenv(name);
    return s ? atoi(s) : dflt;
}

// Pick the tile shape (and K splits for the partial-sum epilogue) with the
// lowest modelled time: full waves of workgroups over 256 CUs, weighted by the
// tile's efficiency, plus the traffic of the fp32 slabs.
Plan make_plan(GemmEpilogue epi, int M, int N, int K)
{
    const int n_out = epi == kEpiSwiglu ? N / 2 : N;
    Plan best{2, 1};
    double best_cost = 1e300;
    const int max_splits = epi == kEpiPartial ? 8 : 1;
    for (int c = 0; c < kNumCfg; ++c) {
        const int bn_out = epi == kEpiSwiglu ? kCfg[c].bn / 2 : kCfg[c].bn;
        const long tiles = (long)((M + kCfg[c].bm - 1) / kCfg[c].bm) * ((n_out + bn_out - 1) / bn_out);
        const int per_cu = (kCfg[c].bm + kCfg[c].bn) * 128 * 2 <= 80 * 1024 ? 2 : 1;  // LDS-limited residency
        for (int s = 1; s <= max_splits; s *= 2) {
            const int kps = ((K + s - 1) / s + kBK - 1) / kBK * kBK;
            if (s > 1 && kps * (s - 1) >= K) continue;
            const long wgs = tiles * s;
            const long waves = (wgs + (long)kNumCU * per_cu - 1) / ((long)kNumCU * per_cu);
            double cost = (double)waves * per_cu * kCfg[c].bm * kCfg[c].bn * (double)kps / kCfg[c].eff;
            cost += 4000.0 * kBK * 64;                                  // prologue / epilogue per launch
            if (epi == kEpiPartial) cost += (double)s * M * N * 40.0;   // slab write + read
            if (cost < best_cost) { best_cost = cost; best = Plan{c, s}; }
        }
    }
    const int fc = env_int("DLLM_GEMM_CFG", -1), fs = env_int("DLLM_GEMM_SPLITS", -1);
    if (fc >= 0 && fc < kNumCfg) best.cfg = fc;
    if (fs >= 1 && epi == kEpiPartial) best.splits = fs;
    return best;
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int EPI>
hipError_t launch_cfg(hipStream_t stream, const void *A, const void *W, void *C, int M, int N, int K, int splits)
{
    constexpr int BN_OUT = EPI == kEpiSwiglu ? BN / 2 : BN;
    const int n_out = EPI == kEpiSwiglu ? N / 2 : N;
    const int num_m = (M + BM - 1) / BM, num_n = (n_out + BN_OUT - 1) / BN_OUT;
    const int kps = ((K + splits - 1) / splits + kBK - 1) / kBK * kBK;
    const size_t lds = (size_t)2 * (BM + BN) * kChunksPerRow * sizeof(uint4);
    auto kern = gemm_kernel<BM, BN, WAVES_M, WAVES_N, EPI>;
    static bool attr_done = false;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    hipLaunchKernelGGL(kern, dim3(num_m * num_n, splits), dim3(kThreads), lds, stream, (const uint16_t *)A,
                       (const uint16_t *)W, C, M, N, K, kps, num_m, num_n);
    return hipGetLastError();
}

template <int EPI>
hipError_t dispatch(hipStream_t stream, Plan p, const void *A, const void *W, void *C, int M, int N, int K)
{
    switch (p.cfg) {
    case 0: return launch_cfg<256, 256, 2, 2, EPI>(stream, A, W, C, M, N, K, p.splits);
    case 1: return launch_cfg<256, 128, 2, 2, EPI>(stream, A, W, C, M, N, K, p.splits);
    case 2: return launch_cfg<128, 128, 2, 2, EPI>(stream, A, W, C, M, N, K, p.splits);
    default: return launch_cfg<128, 64, 4, 1, EPI>(stream, A, W, C, M, N, K, p.splits);
    }
}

}  // namespace

int gemm_num_splits(int M, int N, int K) { return make_plan(kEpiPartial, M, N, K).splits; }

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
