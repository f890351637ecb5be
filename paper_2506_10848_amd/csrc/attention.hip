// Non-causal flash-style attention for gfx950 (every query attends to all L
// keys of its sequence; no mask).
//
// A wave owns 32 queries and walks the keys in tiles of 64.  Both products run
// on the 32x32x16 bf16 MFMA with the queries on the lane axis:
//     S^T = K Q^T          (A = K rows from LDS,  B = Q kept in registers)
//     O^T = V^T P^T        (A = V^T rows from LDS, B = P straight from the S^T
//                           accumulators, no data movement)
// so the running max, the running sum and the rescale factor of a query live in
// the lane that owns it (the two lanes l and l+32 share a query and split the
// keys).  The K index of the second product is a fixed permutation of the keys
// that makes the S^T accumulator layout directly usable as the B operand; the
// V^T fragment is read with the same permutation.  V is transposed on its way
// into LDS.  Softmax runs in fp32 in the exp2 domain.
#include "internal.h"

namespace dllm {

namespace {

constexpr int kKeysPerTile = 64;
constexpr int kVtStride = kKeysPerTile + 4;  // bf16 elements; 136-byte rows keep 8-byte reads conflict-free
constexpr float kLog2e = 1.4426950408889634f;

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v)
{
    union { uint4 u; bf16x8 b; } c;
    c.u = v;
    return c.b;
}

template <int DH, int NWAVES>
__global__ __launch_bounds__(NWAVES * 64) void attention_kernel(const uint16_t *__restrict__ qkv,
                                                                uint16_t *__restrict__ out, int L, int H)
{
    constexpr int NT = NWAVES * 64;
    constexpr int KSTEPS = DH / 16;       // MFMA K steps over the head dimension
    constexpr int DSUB = DH / 32;         // 32-row sub-tiles of O^T
    constexpr int CH = DH / 8;            // 16-byte chunks per K row
    __shared__ uint4 Ks[kKeysPerTile * CH];
    __shared__ __attribute__((aligned(16))) uint16_t Vt[DH * kVtStride];

    const int d = H * DH;
    const size_t ld = (size_t)3 * d;
    const int h = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int l32 = lane & 31, g = lane >> 5;
    const int q0 = blockIdx.x * (NWAVES * 32) + wave * 32;
    const uint16_t *base = qkv + (size_t)b * L * ld;
    const float c = kLog2e / sqrtf((float)DH);

    // Q fragments (B operand): lane (query l32, half g) holds dims t*16 + g*8 .. +8
    bf16x8 qf[KSTEPS];
    {
        const int qrow = min(q0 + l32, L - 1);
        const uint16_t *qp = base + (size_t)qrow * ld + (size_t)h * DH + g * 8;
#pragma unroll
        for (int t = 0; t < KSTEPS; ++t) qf[t] = as_bf16x8(*reinterpret_cast<const uint4 *>(qp + t * 16));
    }

    floatx16 o[DSUB];
#pragma unroll
    for (int i = 0; i < DSUB; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) o[i][e] = 0.0f;
    float m_run = -3.0e38f, l_run = 0.0f;

    const uint16_t *kbase = base + d + (size_t)h * DH;
    const uint16_t *vbase = base + 2 * d + (size_t)h * DH;

    for (int key0 = 0; key0 < L; key0 += kKeysPerTile) {
        __syncthreads();  // previous tile fully consumed
        // K tile: 64 rows x CH chunks, swizzled by row
        for (int idx = tid; idx < kKeysPerTile * CH; idx += NT) {
            const int row = idx / CH, ch = idx % CH;
            const int key = key0 + row;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (key < L) v = *reinterpret_cast<const uint4 *>(kbase + (size_t)key * ld + ch * 8);
            Ks[row * CH + (ch ^ (row & 7))] = v;
        }
        // V tile, transposed: a thread moves a 4-key x 8-dim block
        for (int blk = tid; blk < (kKeysPerTile / 4) * CH; blk += NT) {
            const int kg = blk % (kKeysPerTile / 4), dg = blk / (kKeysPerTile / 4);
            uint4 v[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int key = key0 + kg * 4 + r;
                v[r] = make_uint4(0, 0, 0, 0);
                if (key < L) v[r] = *reinterpret_cast<const uint4 *>(vbase + (size_t)key * ld + dg * 8);
            }
            const uint32_t *w0 = reinterpret_cast<const uint32_t *>(&v[0]);
            const uint32_t *w1 = reinterpret_cast<const uint32_t *>(&v[1]);
            const uint32_t *w2 = reinterpret_cast<const uint32_t *>(&v[2]);
            const uint32_t *w3 = reinterpret_cast<const uint32_t *>(&v[3]);
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
        __syncthreads();

        // S^T for two 32-key sub-tiles
        floatx16 s[2];
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
#pragma unroll
            for (int e = 0; e < 16; ++e) s[sub][e] = 0.0f;
            const int row = sub * 32 + l32;
#pragma unroll
            for (int t = 0; t < KSTEPS; ++t) {
                const bf16x8 kf = as_bf16x8(Ks[row * CH + ((t * 2 + g) ^ (row & 7))]);
                s[sub] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[t], s[sub], 0, 0, 0);
            }
        }
        // keys past the end of the sequence do not exist
        if (key0 + kKeysPerTile > L) {
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
                    union { uint2 h[2]; bf16x8 v; } vf;
                    vf.h[0] = *reinterpret_cast<const uint2 *>(vr);
                    vf.h[1] = *reinterpret_cast<const uint2 *>(vr + 8);
                    o[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf.v, pf.v, o[i], 0, 0, 0);
                }
            }
    }

    const float l_tot = l_run + __shfl_xor(l_run, 32, kWave);
    const float inv = 1.0f / l_tot;
    const int q = q0 + l32;
    if (q < L) {
        uint16_t *op = out + ((size_t)b * L + q) * d + (size_t)h * DH;
#pragma unroll
        for (int i = 0; i < DSUB; ++i)
#pragma unroll
            for (int e4 = 0; e4 < 4; ++e4) {
                const int dim = i * 32 + 8 * e4 + 4 * g;
                uint2 w;
                w.x = pack_bf16x2(o[i][e4 * 4 + 0] * inv, o[i][e4 * 4 + 1] * inv);
                w.y = pack_bf16x2(o[i][e4 * 4 + 2] * inv, o[i][e4 * 4 + 3] * inv);
                *reinterpret_cast<uint2 *>(op + dim) = w;
            }
    }
}

template <int DH>
hipError_t launch_dh(hipStream_t stream, const void *qkv, void *out, int B, int L, int H)
{
    // 4 waves (128 queries) per workgroup when that still fills the chip, else 2
    const long wg4 = (long)((L + 127) / 128) * H * B;
    if (wg4 >= 512) {
        hipLaunchKernelGGL((attention_kernel<DH, 4>), dim3((L + 127) / 128, H, B), dim3(256), 0, stream,
                           (const uint16_t *)qkv, (uint16_t *)out, L, H);
    } else {
        hipLaunchKernelGGL((attention_kernel<DH, 2>), dim3((L + 63) / 64, H, B), dim3(128), 0, stream,
                           (const uint16_t *)qkv, (uint16_t *)out, L, H);
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_attention(hipStream_t stream, const void *qkv, void *out, int B, int L, int H, int dh)
{
    if (dh == 128) return launch_dh<128>(stream, qkv, out, B, L, H);
    if (dh == 64) return launch_dh<64>(stream, qkv, out, B, L, H);
    return hipErrorInvalidValue;
}

}  // namespace dllm
