// Non-causal flash-style attention for gfx950 (every query attends to all L
// keys of its sequence; no mask).
//
// A workgroup has 4 waves of 32 queries each.  With KVSPLIT = 1 they cover 128
// queries and walk all keys together (64 keys per step).  With KVSPLIT = 2 (short
// sequences, few workgroups) waves 0/1 and 2/3 form two halves that walk disjoint
// halves of the key range for the same 64 queries and are merged at the end with
// the log-sum-exp rule, which halves the length of the sequential chain.  Inside a wave (32
// queries) both products run on the 32x32x16 bf16 MFMA with the queries on the
// lane axis:
//     S^T = K Q^T          (A = K rows from LDS,  B = Q kept in registers)
//     O^T = V^T P^T        (A = V^T rows from LDS, B = P straight from the S^T
//                           accumulators, no data movement)
// so the running max, the running sum and the rescale factor of a query live in
// the lane that owns it (lanes l and l+32 share a query and split the keys).
// The K index of the second product is a fixed permutation of the keys that
// makes the S^T accumulator layout directly usable as the B operand; the V^T
// fragment is read with the same permutation.  V is transposed on its way into
// LDS.  The K / V tile of step t+1 is fetched into registers before the math of
// step t, so the global-memory latency hides behind the MFMAs.  Softmax runs in
// fp32 in the exp2 domain.
#include "internal.h"

namespace dllm {

namespace {

constexpr int kKeys = 64;           // keys per step
constexpr int kVtStride = kKeys + 4;  // bf16 elements; 136-byte rows keep the 8-byte fragment reads conflict-free
constexpr float kLog2e = 1.4426950408889634f;
constexpr int kThreads = 256;

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v)
{
    union { uint4 u; bf16x8 b; } c;
    c.u = v;
    return c.b;
}

template <int DH, int KVSPLIT>
struct Smem {
    static constexpr int CH = DH / 8;  // 16-byte chunks per K row
    uint4 Ks[KVSPLIT][kKeys * CH];
    uint16_t Vt[KVSPLIT][DH * kVtStride];
};

// chunk swizzle of a K row: rows of 256 bytes cover all 64 banks, rows of 128
// bytes cover half of them
template <int DH>
__device__ __forceinline__ int k_swz(int row)
{
    return DH == 128 ? (row & 15) : ((row >> 1) & 7);
}

template <int DH, int KVSPLIT>
__global__ __launch_bounds__(kThreads, 2) void attention_kernel(const uint16_t *__restrict__ qsrc,
                                                             const uint16_t *__restrict__ kvsrc,
                                                             uint16_t *__restrict__ out, int L, int H, int nq,
                                                             SeqRows rows, int out_panel_rows)
{
    constexpr int KSTEPS = DH / 16;  // MFMA K steps over the head dimension
    constexpr int DSUB = DH / 32;    // 32-row sub-tiles of O^T
    constexpr int CH = DH / 8;
    constexpr int HT = kThreads / KVSPLIT;             // threads that share one K / V tile
    constexpr int QT = 128 / KVSPLIT;                  // queries per workgroup
    constexpr int K_LOADS = kKeys * CH / HT;           // per thread
    constexpr int V_TOTAL = (kKeys / 4) * CH;          // 4-key x 8-dim blocks of a V tile
    constexpr int V_BLOCKS = (V_TOTAL + HT - 1) / HT;  // per thread
    extern __shared__ uint4 smem_raw[];
    Smem<DH, KVSPLIT> &sm = *reinterpret_cast<Smem<DH, KVSPLIT> *>(smem_raw);

    const int d = H * DH;
    const size_t ld = (size_t)3 * d;
    // Workgroups of one (batch, head) share its K and V: give them ids congruent mod 8, which
    // the dispatcher places on the same XCD, so each K/V tile crosses into one L2 only.
    const int nbh = (int)gridDim.x / nq;
    int qblk, bh;
    {
        const int pid = blockIdx.x, n8 = nbh & ~7, head = nq * n8;
        if (pid < head) {
            const int j = pid >> 3;
            qblk = j % nq;
            bh = (j / nq) * 8 + (pid & 7);
        } else {
            const int r = pid - head;
            qblk = r % nq;
            bh = n8 + r / nq;
        }
    }
    const int h = bh % H, b = bh / H;
    // queries: rows [qfirst, qfirst + Lq) of qsrc; keys and values: the L rows of sequence b in kvsrc
    const int qfirst = rows.first[b], Lq = rows.count[b];
    if (qblk * QT >= Lq) return;  // uniform over the workgroup
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int half = KVSPLIT == 2 ? wave >> 1 : 0, qgroup = KVSPLIT == 2 ? wave & 1 : wave, htid = tid & (HT - 1);
    const int l32 = lane & 31, g = lane >> 5;
    const int q0 = qblk * QT + qgroup * 32;
    const uint16_t *base = kvsrc + (size_t)b * L * ld;
    const float c = kLog2e / sqrtf((float)DH);

    // key steps of this half
    const int ntiles = (L + kKeys - 1) / kKeys;
    const int n_first = KVSPLIT == 2 ? (ntiles + 1) / 2 : ntiles;
    const int my_first = half ? n_first : 0;
    const int my_count = half ? ntiles - n_first : n_first;
    const int iters = n_first;  // both halves loop together

    // Q fragments (B operand): lane (query l32, half g) holds dims t*16 + g*8 .. +8
    bf16x8 qf[KSTEPS];
    {
        const int qrow = qfirst + min(q0 + l32, Lq - 1);
        const uint16_t *qp = qsrc + (size_t)qrow * ld + (size_t)h * DH + g * 8;
#pragma unroll
        for (int t = 0; t < KSTEPS; ++t) qf[t] = as_bf16x8(*reinterpret_cast<const uint4 *>(qp + t * 16));
    }

    const uint16_t *kbase = base + d + (size_t)h * DH;
    const uint16_t *vbase = base + 2 * d + (size_t)h * DH;
    uint4 kreg[K_LOADS], vreg[V_BLOCKS][4];

    const char *kbytes = reinterpret_cast<const char *>(kbase), *vbytes = reinterpret_cast<const char *>(vbase);
    const uint32_t ldb = (uint32_t)ld * 2u;  // 32-bit byte offsets from the sequence base
    auto fetch = [&](int it) {  // step `it` of this half -> registers (zeros past the end)
        const int key0 = (my_first + it) * kKeys;
        const bool live = it < my_count;
#pragma unroll
        for (int t = 0; t < K_LOADS; ++t) {
            const int idx = htid + t * HT, row = idx / CH, ch = idx % CH;
            const int key = key0 + row;
            kreg[t] = (live && key < L) ? *reinterpret_cast<const uint4 *>(kbytes + ((uint32_t)key * ldb + (uint32_t)ch * 16u))
                                        : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int t = 0; t < V_BLOCKS; ++t) {
            const int blk = htid + t * HT, kg = blk % (kKeys / 4), dg = blk / (kKeys / 4);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int key = key0 + kg * 4 + r;
                vreg[t][r] = (live && key < L && blk < V_TOTAL) ? *reinterpret_cast<const uint4 *>(vbytes + ((uint32_t)key * ldb + (uint32_t)dg * 16u))
                                               : make_uint4(0, 0, 0, 0);
            }
        }
    };
    auto stash = [&]() {  // registers -> LDS of this half: K swizzled, V transposed
        uint4 *Ks = sm.Ks[half];
        uint16_t *Vt = sm.Vt[half];
#pragma unroll
        for (int t = 0; t < K_LOADS; ++t) {
            const int idx = htid + t * HT, row = idx / CH, ch = idx % CH;
            Ks[row * CH + (ch ^ k_swz<DH>(row))] = kreg[t];
        }
#pragma unroll
        for (int t = 0; t < V_BLOCKS; ++t) {
            const int blk = htid + t * HT, kg = blk % (kKeys / 4), dg = blk / (kKeys / 4);
            if (blk >= V_TOTAL) continue;
            const uint32_t *w0 = reinterpret_cast<const uint32_t *>(&vreg[t][0]);
            const uint32_t *w1 = reinterpret_cast<const uint32_t *>(&vreg[t][1]);
            const uint32_t *w2 = reinterpret_cast<const uint32_t *>(&vreg[t][2]);
            const uint32_t *w3 = reinterpret_cast<const uint32_t *>(&vreg[t][3]);
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                // dims 2p (low halves) and 2p+1 (high halves) of the four keys
                uint2 lo, hi;
                lo.x = (w0[p] & 0xffffu) | (w1[p] << 16);
                lo.y = (w2[p] & 0xffffu) | (w3[p] << 16);
                hi.x = (w0[p] >> 16) | (w1[p] & 0xffff0000u);
                hi.y = (w2[p] >> 16) | (w3[p] & 0xffff0000u);
                *reinterpret_cast<uint2 *>(&Vt[(dg * 8 + 2 * p) * kVtStride + kg * 4]) = lo;
                *reinterpret_cast<uint2 *>(&Vt[(dg * 8 + 2 * p + 1) * kVtStride + kg * 4]) = hi;
            }
        }
    };

    floatx16 o[DSUB];
#pragma unroll
    for (int i = 0; i < DSUB; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) o[i][e] = 0.0f;
    float m_run = -3.0e38f, l_run = 0.0f;

    fetch(0);
    stash();
    __syncthreads();

    for (int it = 0; it < iters; ++it) {
        if (it + 1 < iters) fetch(it + 1);
        if (it < my_count) {
            const int key0 = (my_first + it) * kKeys;
            const uint4 *Ks = sm.Ks[half];
            const uint16_t *Vt = sm.Vt[half];
            // S^T for two 32-key sub-tiles
            floatx16 s[2];
#pragma unroll
            for (int sub = 0; sub < 2; ++sub) {
#pragma unroll
                for (int e = 0; e < 16; ++e) s[sub][e] = 0.0f;
                const int row = sub * 32 + l32;
                const int swz = k_swz<DH>(row);
#pragma unroll
                for (int t = 0; t < KSTEPS; ++t) {
                    const bf16x8 kf = as_bf16x8(Ks[row * CH + ((t * 2 + g) ^ swz)]);
                    s[sub] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[t], s[sub], 0, 0, 0);
                }
            }
            // keys past the end of the sequence do not exist
            if (key0 + kKeys > L) {
#pragma unroll
                for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const int key = key0 + sub * 32 + 8 * (e / 4) + 4 * g + (e % 4);
                        if (key >= L) s[sub][e] = -INFINITY;
                    }
            }
            // online softmax for this lane's query
            float mt = s[0][0];
#pragma unroll
            for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                for (int e = 0; e < 16; ++e) mt = fmaxf(mt, s[sub][e]);
            mt = fmaxf(mt, __shfl_xor(mt, 32, kWave));
            const float m_new = fmaxf(m_run, mt);
            const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c);
            const float off = -m_new * c;
            float psum = 0.0f;
#pragma unroll
            for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const float p = __builtin_amdgcn_exp2f(fmaf(s[sub][e], c, off));
                    s[sub][e] = p;
                    psum += p;
                }
            l_run = l_run * alpha + psum;
            m_run = m_new;
#pragma unroll
            for (int i = 0; i < DSUB; ++i)
#pragma unroll
                for (int e = 0; e < 16; ++e) o[i][e] *= alpha;

            // O^T += V^T P^T, 16 keys per MFMA
#pragma unroll
            for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) {
                    union { uint4 u; bf16x8 v; } pf;
                    pf.u.x = pack_bf16x2(s[sub][kb * 8 + 0], s[sub][kb * 8 + 1]);
                    pf.u.y = pack_bf16x2(s[sub][kb * 8 + 2], s[sub][kb * 8 + 3]);
                    pf.u.z = pack_bf16x2(s[sub][kb * 8 + 4], s[sub][kb * 8 + 5]);
                    pf.u.w = pack_bf16x2(s[sub][kb * 8 + 6], s[sub][kb * 8 + 7]);
                    const int kcol = sub * 32 + kb * 16 + 4 * g;  // keys kcol..+3 and kcol+8..+11
#pragma unroll
                    for (int i = 0; i < DSUB; ++i) {
                        const uint16_t *vr = &Vt[(i * 32 + l32) * kVtStride + kcol];
                        union { uint2 h2[2]; bf16x8 v; } vf;
                        vf.h2[0] = *reinterpret_cast<const uint2 *>(vr);
                        vf.h2[1] = *reinterpret_cast<const uint2 *>(vr + 8);
                        o[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf.v, pf.v, o[i], 0, 0, 0);
                    }
                }
        }
        __syncthreads();  // everyone is done with this step's tiles
        if (it + 1 < iters) stash();
        __syncthreads();
    }

    // ---- merge the two halves (log-sum-exp), normalise, store ----------------
    float l_tot = l_run + __shfl_xor(l_run, 32, kWave);
    float a0 = 1.0f, a1 = 0.0f, l1 = 0.0f;
    float *xo = reinterpret_cast<float *>(smem_raw);       // [qgroup][DSUB*16][64 lanes]
    float *xs = xo + 2 * DSUB * 16 * 64;                    // [qgroup][2][64 lanes]: m, l
    if (KVSPLIT == 2) {
        if (half == 1) {
#pragma unroll
            for (int i = 0; i < DSUB; ++i)
#pragma unroll
                for (int e = 0; e < 16; ++e) xo[(qgroup * DSUB * 16 + i * 16 + e) * 64 + lane] = o[i][e];
            xs[(qgroup * 2 + 0) * 64 + lane] = m_run;
            xs[(qgroup * 2 + 1) * 64 + lane] = l_tot;
        }
        __syncthreads();
        if (half == 1) return;
        const float m1 = xs[(qgroup * 2 + 0) * 64 + lane];
        l1 = xs[(qgroup * 2 + 1) * 64 + lane];
        const float m = fmaxf(m_run, m1);
        a0 = __builtin_amdgcn_exp2f((m_run - m) * c);
        a1 = __builtin_amdgcn_exp2f((m1 - m) * c);
    }
    const float inv = 1.0f / (l_tot * a0 + l1 * a1);
    const int q = q0 + l32;
    if (q < Lq) {
        // row-major: out[row][h * DH + dim]; panel-major: panel (h * DH + dim) / 32, 32 elements per row
        const size_t orow = (size_t)qfirst + q;
        uint16_t *op = out_panel_rows ? out + (((size_t)h * (DH / 32)) * out_panel_rows + orow) * 32
                                      : out + orow * d + (size_t)h * DH;
        const size_t sub_pitch = out_panel_rows ? (size_t)out_panel_rows * 32 - 32 : 0;  // added per 32-dim sub-tile
#pragma unroll
        for (int i = 0; i < DSUB; ++i)
#pragma unroll
            for (int e4 = 0; e4 < 4; ++e4) {
                float y[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float v = o[i][e4 * 4 + e] * a0;
                    if (KVSPLIT == 2) v += xo[(qgroup * DSUB * 16 + i * 16 + e4 * 4 + e) * 64 + lane] * a1;
                    y[e] = v * inv;
                }
                const int dim = i * 32 + 8 * e4 + 4 * g;
                uint2 w;
                w.x = pack_bf16x2(y[0], y[1]);
                w.y = pack_bf16x2(y[2], y[3]);
                *reinterpret_cast<uint2 *>(op + dim + i * sub_pitch) = w;
            }
    }
}

template <int DH, int KVSPLIT>
hipError_t launch_split(hipStream_t stream, const void *q, const void *kv, void *out, int B, int Lk, int H,
                        const SeqRows &rows, int max_count, int out_panel_rows)
{
    constexpr int QT = 128 / KVSPLIT;
    const size_t lds = sizeof(Smem<DH, KVSPLIT>);
    static_assert(KVSPLIT == 1 || sizeof(Smem<DH, 2>) >= (2 * (DH / 32) * 16 * 64 + 4 * 64) * sizeof(float),
                  "merge buffer fits");
    auto kern = attention_kernel<DH, KVSPLIT>;
    // once per kernel, whichever thread comes first (initialisation of a local static is thread-safe)
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (attr != hipSuccess) return attr;
    const int nq = (max_count + QT - 1) / QT;
    hipLaunchKernelGGL(kern, dim3(nq * H * B), dim3(kThreads), lds, stream, (const uint16_t *)q, (const uint16_t *)kv,
                       (uint16_t *)out, Lk, H, nq, rows, out_panel_rows);
    return hipGetLastError();
}

template <int DH>
hipError_t launch_dh(hipStream_t stream, const void *q, const void *kv, void *out, int B, int Lk, int H,
                     const SeqRows &rows, int out_panel_rows)
{
    int max_count = 0;
    for (int b = 0; b < B; ++b) max_count = rows.count[b] > max_count ? rows.count[b] : max_count;
    if (max_count == 0) return hipSuccess;
    // few workgroups: split the keys inside a workgroup to shorten the chain
    const long wgs128 = (long)((max_count + 127) / 128) * H * B;
    if (wgs128 < 1024) return launch_split<DH, 2>(stream, q, kv, out, B, Lk, H, rows, max_count, out_panel_rows);
    return launch_split<DH, 1>(stream, q, kv, out, B, Lk, H, rows, max_count, out_panel_rows);
}

}  // namespace

hipError_t launch_attention_rows(hipStream_t stream, const void *q, const void *kv, void *out, int B, int Lk, int H,
                                 int dh, const SeqRows &rows, int out_panel_rows)
{
    if (B < 1 || B > DLLM_MAX_BATCH) return hipErrorInvalidValue;
    if (dh == 128) return launch_dh<128>(stream, q, kv, out, B, Lk, H, rows, out_panel_rows);
    if (dh == 64) return launch_dh<64>(stream, q, kv, out, B, Lk, H, rows, out_panel_rows);
    return hipErrorInvalidValue;
}

hipError_t launch_attention(hipStream_t stream, const void *qkv, void *out, int B, int L, int H, int dh,
                            int out_panel_rows)
{
    if (B <= DLLM_MAX_BATCH) {
        SeqRows rows;
        for (int b = 0; b < B; ++b) { rows.first[b] = b * L; rows.count[b] = L; }
        return launch_attention_rows(stream, qkv, qkv, out, B, L, H, dh, rows, out_panel_rows);
    }
    if (out_panel_rows) return hipErrorInvalidValue;
    // more sequences than the row table holds (test hook only): one launch per group
    for (int b0 = 0; b0 < B; b0 += DLLM_MAX_BATCH) {
        const int nb = B - b0 < DLLM_MAX_BATCH ? B - b0 : DLLM_MAX_BATCH;
        const size_t off = (size_t)b0 * L * 3 * H * dh;
        hipError_t e = launch_attention(stream, (const uint16_t *)qkv + off,
                                        (uint16_t *)out + (size_t)b0 * L * H * dh, nb, L, H, dh);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace dllm
