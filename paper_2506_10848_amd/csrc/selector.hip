// Selector kernels: the per-position greedy decode + confidence ("row phase",
// Section 3.1 eq. 3 and the confidence equation) and the per-sequence SlowFast
// selection rule with the state transition ("sequence phase", Section 3.3,
// eqs. 6 and 9, Algorithm 1's cautious-decoding / in-span / fallback branches).
//
// Row phase: HBM-bound.  One 256-thread workgroup streams one bf16 logits row
// with 16-byte loads, four in flight per lane, and keeps a running
// (max, sum of exp, first chunk holding the max) per lane; lanes are merged
// with the log-sum-exp rule.  Rows that are not masked or lie outside their
// sequence's window are never read.
//
// Sequence phase: one workgroup per sequence over L positions in LDS.
#include "internal.h"

namespace dllm {

namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kNegBig = -3.0e38f;
constexpr int kRowThreads = 256;

struct RowAcc {
    float m;  // running max
    float s;  // sum of exp(x - m)
    int c;    // lowest chunk (or element) index where m was seen
};

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ RowAcc combine(RowAcc a, RowAcc b)
{
    RowAcc r;
    r.m = fmaxf(a.m, b.m);
    r.s = a.s * fast_exp2((a.m - r.m) * kLog2e) + b.s * fast_exp2((b.m - r.m) * kLog2e);
    bool take_a = (a.m > b.m) || (a.m == b.m && a.c < b.c);
    r.c = take_a ? a.c : b.c;
    return r;
}

// Fold NK 16-byte chunks (8 bf16 each) into the accumulator.  chunk0 is the
// index of this lane's first chunk; consecutive chunks are `stride` apart.
template <int NK>
__device__ __forceinline__ void fold_chunks(RowAcc &acc, const u32x4 *q, int chunk0, int stride, int mask_chunk,
                                            int mask_j)
{
    float x[NK][8];
#pragma unroll
    for (int k = 0; k < NK; ++k) {
        x[k][0] = bf16_lo(q[k].x); x[k][1] = bf16_hi(q[k].x);
        x[k][2] = bf16_lo(q[k].y); x[k][3] = bf16_hi(q[k].y);
        x[k][4] = bf16_lo(q[k].z); x[k][5] = bf16_hi(q[k].z);
        x[k][6] = bf16_lo(q[k].w); x[k][7] = bf16_hi(q[k].w);
    }
    // the [MASK] id is not a legal prediction: drop it from max and sum
#pragma unroll
    for (int k = 0; k < NK; ++k)
        if (chunk0 + k * stride == mask_chunk) {
#pragma unroll
            for (int j = 0; j < 8; ++j) x[k][j] = (j == mask_j) ? -INFINITY : x[k][j];
        }
    float cm[NK];
#pragma unroll
    for (int k = 0; k < NK; ++k) {
        float a = fmaxf(fmaxf(x[k][0], x[k][1]), fmaxf(x[k][2], x[k][3]));
        float b = fmaxf(fmaxf(x[k][4], x[k][5]), fmaxf(x[k][6], x[k][7]));
        cm[k] = fmaxf(a, b);
    }
    float gm = cm[0];
#pragma unroll
    for (int k = 1; k < NK; ++k) gm = fmaxf(gm, cm[k]);
    int kb = NK - 1;
#pragma unroll
    for (int k = NK - 2; k >= 0; --k) kb = (cm[k] == gm) ? k : kb;  // earliest chunk holding gm
    acc.c = (gm > acc.m) ? chunk0 + kb * stride : acc.c;
    float mn = fmaxf(acc.m, gm);
    float off = -mn * kLog2e;
    float s = acc.s * fast_exp2((acc.m - mn) * kLog2e);
#pragma unroll
    for (int k = 0; k < NK; ++k)
#pragma unroll
        for (int j = 0; j < 8; ++j) s += fast_exp2(fmaf(x[k][j], kLog2e, off));
    acc.s = s;
    acc.m = mn;
}

__device__ __forceinline__ RowAcc block_reduce(RowAcc acc)
{
    __shared__ RowAcc part[kRowThreads / kWave];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        RowAcc other;
        other.m = __shfl_xor(acc.m, o, kWave);
        other.s = __shfl_xor(acc.s, o, kWave);
        other.c = __shfl_xor(acc.c, o, kWave);
        acc = combine(acc, other);
    }
    const int wave = threadIdx.x / kWave;
    if ((threadIdx.x & (kWave - 1)) == 0) part[wave] = acc;
    __syncthreads();
    RowAcc r = part[0];
#pragma unroll
    for (int w = 1; w < kRowThreads / kWave; ++w) r = combine(r, part[w]);
    return r;
}

// VEC: V % 8 == 0 and the logits base is 16-byte aligned, so every row is.
template <bool VEC>
__global__ __launch_bounds__(kRowThreads) void row_phase_kernel(const uint16_t *__restrict__ logits, int L, int V,
                                                                int mask_id, const uint8_t *__restrict__ mask,
                                                                SelectArgs args, int32_t *__restrict__ pred,
                                                                float *__restrict__ conf)
{
    const int r = blockIdx.x;
    const int b = r / L, i = r - b * L;
    const SeqWindow w = args.w[b];
    if (i < w.lo || i > w.eval_hi || mask[r] == 0) return;  // uniform over the block

    const uint16_t *row = logits + (size_t)r * V;
    const int tid = threadIdx.x;
    RowAcc acc{kNegBig, 0.0f, 0x7fffffff};

    if (VEC) {
        const u32x4 *p = reinterpret_cast<const u32x4 *>(row);
        const int nchunks = V >> 3;
        const int mask_chunk = mask_id >> 3, mask_j = mask_id & 7;
        constexpr int NK = 4;
        int c = tid;
        for (; c + (NK - 1) * kRowThreads < nchunks; c += NK * kRowThreads) {
            u32x4 q[NK];
#pragma unroll
            for (int k = 0; k < NK; ++k) q[k] = __builtin_nontemporal_load(p + c + k * kRowThreads);
            fold_chunks<NK>(acc, q, c, kRowThreads, mask_chunk, mask_j);
        }
        for (; c < nchunks; c += kRowThreads) {
            u32x4 q[1];
            q[0] = __builtin_nontemporal_load(p + c);
            fold_chunks<1>(acc, q, c, kRowThreads, mask_chunk, mask_j);
        }
    } else {
        for (int v = tid; v < V; v += kRowThreads) {
            if (v == mask_id) continue;
            float x = bf16_bits_to_float(row[v]);
            if (x > acc.m) {
                acc.s = acc.s * fast_exp2((acc.m - x) * kLog2e);
                acc.m = x;
                acc.c = v;
            }
            acc.s += fast_exp2((x - acc.m) * kLog2e);
        }
    }

    RowAcc tot = block_reduce(acc);
    if (tid == 0) {
        int arg = tot.c;
        if (VEC) {
            // lowest id inside the winning chunk that equals the max
            const uint16_t *e = row + (size_t)tot.c * 8;
            int base = tot.c * 8;
            arg = -1;
            for (int j = 7; j >= 0; --j)
                if (base + j != mask_id && bf16_bits_to_float(e[j]) == tot.m) arg = base + j;
        }
        pred[r] = arg;
        conf[r] = 1.0f / tot.s;
    }
}

// Row phase after a vocabulary projection with the row-statistics epilogue: the statistics of
// `parts` column slices per row, planes of [parts][n_rows] (max, sum of exp(x - max), lowest
// column holding the max), are merged with the same log-sum-exp rule.  Row lr of the planes is
// batch row first_row + lr.
__global__ __launch_bounds__(kRowThreads) void rowstats_merge_kernel(const float *__restrict__ stats, int parts,
                                                                     int n_rows, int first_row, int L,
                                                                     const uint8_t *__restrict__ mask, SelectArgs args,
                                                                     int32_t *__restrict__ pred, float *__restrict__ conf)
{
    const int lr = blockIdx.x, r = first_row + lr;
    const int b = r / L, i = r - b * L;
    const SeqWindow w = args.w[b];
    if (i < w.lo || i > w.eval_hi || mask[r] == 0) return;  // uniform over the block
    const size_t plane = (size_t)parts * n_rows;
    const int *cols = reinterpret_cast<const int *>(stats) + 2 * plane;
    RowAcc acc{kNegBig, 0.0f, 0x7fffffff};
    for (int p = threadIdx.x; p < parts; p += kRowThreads) {
        const size_t at = (size_t)p * n_rows + lr;
        acc = combine(acc, RowAcc{stats[at], stats[plane + at], cols[at]});
    }
    const RowAcc tot = block_reduce(acc);
    if (threadIdx.x == 0) {
        pred[r] = tot.c;
        conf[r] = 1.0f / tot.s;
    }
}

// ---- sequence phase ---------------------------------------------------------

constexpr int kSeqThreads = 512;

__device__ __forceinline__ int block_exclusive_scan(int f, int *wave_tot, int &total)
{
    // f is 0/1 per thread
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    unsigned long long bal = __ballot(f);
    int excl = __popcll(bal & ((1ull << lane) - 1ull));
    if (lane == 0) wave_tot[wave] = __popcll(bal);
    __syncthreads();
    int off = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < kSeqThreads / kWave; ++w) {
        int t = wave_tot[w];
        off += (w < wave) ? t : 0;
        tot += t;
    }
    __syncthreads();
    total = tot;
    return off + excl;
}

__global__ __launch_bounds__(kSeqThreads) void seq_phase_kernel(int L, int32_t *__restrict__ tokens,
                                                                uint8_t *__restrict__ mask,
                                                                int32_t *__restrict__ prev_pred,
                                                                const int32_t *__restrict__ pred,
                                                                const float *__restrict__ conf, SelectArgs args,
                                                                CommitOut out)
{
    extern __shared__ unsigned long long keys[];          // [L] (confidence bits, ~position) of candidates
    uint8_t *flag = reinterpret_cast<uint8_t *>(keys + L);  // [L] 1 = commit
    __shared__ int s_ecand, s_first, s_nhigh, s_ncand, s_nmask, s_count;
    __shared__ unsigned long long s_best;
    __shared__ int wave_tot[kSeqThreads / kWave];

    const int b = blockIdx.x, tid = threadIdx.x;
    const SeqWindow w = args.w[b];
    const size_t row0 = (size_t)b * L;
    if (tid == 0) {
        s_ecand = -1; s_first = 0x7fffffff; s_nhigh = 0; s_ncand = 0; s_nmask = 0; s_best = 0ull;
    }
    __syncthreads();

    int my_masks = 0;
    for (int i = tid; i < L; i += kSeqThreads) {
        const bool m = mask[row0 + i] != 0;
        my_masks += m;
        flag[i] = 0;
        if (m && i > w.hi && i <= w.eval_hi) prev_pred[row0 + i] = pred[row0 + i];  // evaluated, not decided on
        if (m && i >= w.lo && i <= w.hi) {
            const float c = conf[row0 + i];
            const int p = pred[row0 + i];
            if (c > w.tau_min) atomicMax(&s_ecand, i);                       // eq. 6
            atomicMin(&s_first, i);
            const bool high = w.stage == DLLM_STAGE_FAST && c > w.tau_high &&  // eq. 9
                              (w.conv_mode == 0 || p == prev_pred[row0 + i]);
            if (high) { flag[i] = 1; atomicAdd(&s_nhigh, 1); }
            prev_pred[row0 + i] = p;
            const int idx = atomicAdd(&s_ncand, 1);
            keys[idx] = ((unsigned long long)__float_as_uint(c) << 32) | (unsigned)(0xffffffffu - (unsigned)i);
        }
    }
    if (my_masks) atomicAdd(&s_nmask, my_masks);
    __syncthreads();

    const int ncand = s_ncand;
    const bool use_topk = w.stage == DLLM_STAGE_SLOW || (w.stage == DLLM_STAGE_FAST && s_nhigh == 0);
    if (use_topk && ncand > 0) {
        if (w.top_k >= ncand) {
            for (int idx = tid; idx < ncand; idx += kSeqThreads) flag[0xffffffffu - (unsigned)keys[idx]] = 1;
        } else if (w.top_k == 1) {
            unsigned long long best = 0ull;
            for (int idx = tid; idx < ncand; idx += kSeqThreads) best = keys[idx] > best ? keys[idx] : best;
            atomicMax(&s_best, best);
            __syncthreads();
            if (tid == 0) flag[0xffffffffu - (unsigned)s_best] = 1;
        } else if (ncand <= 1024) {
            // rank by counting: keys are distinct, so exactly top_k ranks fall below top_k
            for (int idx = tid; idx < ncand; idx += kSeqThreads) {
                const unsigned long long key = keys[idx];
                int rank = 0;
                for (int j = 0; j < ncand; ++j) rank += keys[j] > key;
                if (rank < w.top_k) flag[0xffffffffu - (unsigned)key] = 1;
            }
        } else {
            // many candidates: the top_k-th largest key, bit by bit from the top (the largest value t such
            // that at least top_k keys are >= t); 64 counting passes over the keys instead of ncand per key
            unsigned long long t = 0ull;
            for (int bit = 63; bit >= 0; --bit) {
                const unsigned long long cand = t | (1ull << bit);
                if (tid == 0) s_count = 0;
                __syncthreads();
                int mine = 0;
                for (int idx = tid; idx < ncand; idx += kSeqThreads) mine += keys[idx] >= cand;
                if (mine) atomicAdd(&s_count, mine);
                __syncthreads();
                if (s_count >= w.top_k) t = cand;   // uniform over the workgroup
                __syncthreads();
            }
            for (int idx = tid; idx < ncand; idx += kSeqThreads)
                if (keys[idx] >= t) flag[0xffffffffu - (unsigned)keys[idx]] = 1;
        }
    }
    __syncthreads();

    // ordered compaction of the commit flags + the transition
    int base = 0;
    const int lo = w.lo < 0 ? 0 : w.lo, hi = w.hi >= L ? L - 1 : w.hi;
    for (int start = lo; start <= hi; start += kSeqThreads) {
        const int i = start + tid;
        const int f = (i <= hi) ? flag[i] : 0;
        int total;
        const int slot = base + block_exclusive_scan(f, wave_tot, total);
        if (f) {
            const int p = pred[row0 + i];
            if (slot < out.capacity) {
                const size_t o = (size_t)b * out.capacity + slot;
                out.pos[o] = i;
                out.tok[o] = p;
                out.conf[o] = conf[row0 + i];
            }
            tokens[row0 + i] = p;
            mask[row0 + i] = 0;
        }
        base += total;
    }
    if (tid == 0) {
        out.n_commit[b] = base;
        out.e_cand[b] = s_ecand;
        out.first_masked[b] = s_first == 0x7fffffff ? -1 : s_first;
        out.n_masked_after[b] = s_nmask - base;
    }
}

}  // namespace

hipError_t launch_row_phase(hipStream_t stream, const void *logits, int B, int L, int V, int mask_id,
                            const uint8_t *mask, const SelectArgs &args, int32_t *pred, float *conf)
{
    const bool vec = (V % 8 == 0) && ((reinterpret_cast<uintptr_t>(logits) & 15) == 0);
    dim3 grid(B * L), block(kRowThreads);
    if (vec)
        hipLaunchKernelGGL(row_phase_kernel<true>, grid, block, 0, stream, (const uint16_t *)logits, L, V, mask_id,
                           mask, args, pred, conf);
    else
        hipLaunchKernelGGL(row_phase_kernel<false>, grid, block, 0, stream, (const uint16_t *)logits, L, V, mask_id,
                           mask, args, pred, conf);
    return hipGetLastError();
}

hipError_t launch_rowstats_merge(hipStream_t stream, const float *stats, int parts, int n_rows, int first_row, int L,
                                 const uint8_t *mask, const SelectArgs &args, int32_t *pred, float *conf)
{
    hipLaunchKernelGGL(rowstats_merge_kernel, dim3(n_rows), dim3(kRowThreads), 0, stream, stats, parts, n_rows,
                       first_row, L, mask, args, pred, conf);
    return hipGetLastError();
}

hipError_t launch_seq_phase(hipStream_t stream, int B, int L, int32_t *tokens, uint8_t *mask, int32_t *prev_pred,
                            const int32_t *pred, const float *conf, const SelectArgs &args, const CommitOut &out)
{
    const size_t lds = (size_t)L * 9 + 16;
    // once, whichever thread comes first (initialisation of a local static is thread-safe)
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(seq_phase_kernel),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, 8192 * 9 + 16);
    if (attr != hipSuccess) return attr;
    hipLaunchKernelGGL(seq_phase_kernel, dim3(B), dim3(kSeqThreads), lds, stream, L, tokens, mask, prev_pred, pred,
                       conf, args, out);
    return hipGetLastError();
}

}  // namespace dllm
