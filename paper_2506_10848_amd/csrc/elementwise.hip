// Memory-bound pieces of the forward pass: embedding gather, residual-add +
// RMSNorm (which also sums the fp32 split-K slabs of the preceding GEMM), and
// rotate-half RoPE on the q and k thirds of the fused qkv activations.
#include "internal.h"

namespace dllm {

namespace {

constexpr int kThreads = 256;

// x[r][:] = float(E[tokens[r]][:]); d % 8 == 0.  An id outside [0, vocab) is never used as an index:
// its row becomes zeros and *bad_token is set to 1 (the host reports it at its next synchronisation).
// With gain != null the kernel also leaves what the first projection needs to apply the first RMSNorm
// itself: h[r][:] = bf16(x[r][:] * gain[:]) (row-major, or panel-major with h_panel_rows rows per panel)
// and ssq[r * ssq_stride] = sum of x[r][:]^2.
__global__ __launch_bounds__(kThreads) void embed_kernel(const int32_t *__restrict__ tokens,
                                                         const int32_t *__restrict__ rows,
                                                         const uint16_t *__restrict__ E, float *__restrict__ x, int d,
                                                         int vocab, int32_t *__restrict__ bad_token,
                                                         const uint16_t *__restrict__ gain, uint16_t *__restrict__ h,
                                                         int h_panel_rows, float *__restrict__ ssq, int ssq_stride)
{
    __shared__ float wsum[kThreads / kWave];
    const int r = blockIdx.x;
    const int tok = tokens[rows ? rows[r] : r];
    const bool bad = (unsigned)tok >= (unsigned)vocab;  // uniform over the workgroup
    float4 *dst = reinterpret_cast<float4 *>(x + (size_t)r * d);
    const uint4 *src = reinterpret_cast<const uint4 *>(E + (size_t)(bad ? 0 : tok) * d);
    if (bad && threadIdx.x == 0 && bad_token) *bad_token = 1;
    float ss = 0.0f;
    for (int c = threadIdx.x; c < d / 8; c += kThreads) {
        const uint4 q = bad ? make_uint4(0, 0, 0, 0) : src[c];
        const float4 lo = make_float4(bf16_lo(q.x), bf16_hi(q.x), bf16_lo(q.y), bf16_hi(q.y));
        const float4 hi = make_float4(bf16_lo(q.z), bf16_hi(q.z), bf16_lo(q.w), bf16_hi(q.w));
        dst[2 * c] = lo;
        dst[2 * c + 1] = hi;
        if (gain) {
            ss += lo.x * lo.x + lo.y * lo.y + lo.z * lo.z + lo.w * lo.w + hi.x * hi.x + hi.y * hi.y + hi.z * hi.z + hi.w * hi.w;
            const uint4 g = reinterpret_cast<const uint4 *>(gain)[c];
            uint4 o;
            o.x = pack_bf16x2(lo.x * bf16_lo(g.x), lo.y * bf16_hi(g.x));
            o.y = pack_bf16x2(lo.z * bf16_lo(g.y), lo.w * bf16_hi(g.y));
            o.z = pack_bf16x2(hi.x * bf16_lo(g.z), hi.y * bf16_hi(g.z));
            o.w = pack_bf16x2(hi.z * bf16_lo(g.w), hi.w * bf16_hi(g.w));
            // elements 8c .. 8c+7 of row r: panel c / 4, 16-byte slot c % 4 of the row's 64 bytes
            if (h_panel_rows) reinterpret_cast<uint4 *>(h)[((size_t)(c >> 2) * h_panel_rows + r) * 4 + (c & 3)] = o;
            else reinterpret_cast<uint4 *>(h + (size_t)r * d)[c] = o;
        }
    }
    if (!gain) return;
    ss = wave_sum(ss);
    if ((threadIdx.x & (kWave - 1)) == 0) wsum[threadIdx.x / kWave] = ss;
    __syncthreads();
    if (threadIdx.x == 0) {
        float tot = 0.0f;
#pragma unroll
        for (int w = 0; w < kThreads / kWave; ++w) tot += wsum[w];
        ssq[(size_t)r * ssq_stride] = tot;
    }
}

// dst[rows[r]][d .. 3d) = src[r][d .. 3d), rows of 3d bf16; d % 8 == 0.
__global__ __launch_bounds__(kThreads) void scatter_kv_kernel(const uint16_t *__restrict__ src,
                                                              uint16_t *__restrict__ dst,
                                                              const int32_t *__restrict__ rows, int d)
{
    const int r = blockIdx.x;
    const uint4 *s = reinterpret_cast<const uint4 *>(src + (size_t)r * 3 * d + d);
    uint4 *t = reinterpret_cast<uint4 *>(dst + (size_t)rows[r] * 3 * d + d);
    for (int c = threadIdx.x; c < 2 * d / 8; c += kThreads) t[c] = s[c];
}

// x += sum_s partials[s];  h = bf16( x * rsqrt(mean(x^2) + eps) * gain ).  d % 4 == 0.
// h_panel_rows != 0: h is written panel-major, [d / 32][h_panel_rows][32] (the layout the GEMMs copy fastest).
__global__ __launch_bounds__(kThreads) void add_rmsnorm_kernel(float *__restrict__ x,
                                                               const float *__restrict__ partials, int n_partials,
                                                               size_t slab, const uint16_t *__restrict__ gain,
                                                               uint16_t *__restrict__ h, int d, float eps,
                                                               int h_panel_rows)
{
    __shared__ float wsum[kThreads / kWave];
    const int r = blockIdx.x;
    float4 *xr = reinterpret_cast<float4 *>(x + (size_t)r * d);
    float ss = 0.0f;
    for (int c = threadIdx.x; c < d / 4; c += kThreads) {
        float4 v = xr[c];
        // all slab loads are issued before the first add (a loop of unknown length would take them one
        // latency at a time); the order of the additions stays s = 0, 1, ...
        constexpr int kMaxPartials = 8;
        float4 p[kMaxPartials];
#pragma unroll
        for (int s = 0; s < kMaxPartials; ++s)
            if (s < n_partials) p[s] = reinterpret_cast<const float4 *>(partials + s * slab + (size_t)r * d)[c];
#pragma unroll
        for (int s = 0; s < kMaxPartials; ++s)
            if (s < n_partials) { v.x += p[s].x; v.y += p[s].y; v.z += p[s].z; v.w += p[s].w; }
        if (n_partials) xr[c] = v;
        ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
    }
    ss = wave_sum(ss);
    if ((threadIdx.x & (kWave - 1)) == 0) wsum[threadIdx.x / kWave] = ss;
    __syncthreads();
    float tot = 0.0f;
#pragma unroll
    for (int w = 0; w < kThreads / kWave; ++w) tot += wsum[w];
    const float inv = rsqrtf(tot / (float)d + eps);
    uint2 *hr = reinterpret_cast<uint2 *>(h + (size_t)r * d);
    const uint2 *gr = reinterpret_cast<const uint2 *>(gain);
    for (int c = threadIdx.x; c < d / 4; c += kThreads) {
        const float4 v = xr[c];  // this thread wrote it above
        const uint2 g = gr[c];
        uint2 o;
        o.x = pack_bf16x2(v.x * inv * bf16_lo(g.x), v.y * inv * bf16_hi(g.x));
        o.y = pack_bf16x2(v.z * inv * bf16_lo(g.y), v.w * inv * bf16_hi(g.y));
        if (h_panel_rows)  // elements 4c .. 4c+3 of row r: panel c / 8, 8-byte slot c % 8 of the row's 64 bytes
            reinterpret_cast<uint2 *>(h)[((size_t)(c >> 3) * h_panel_rows + r) * 8 + (c & 7)] = o;
        else
            hr[c] = o;
    }
}

// (cos, sin) of pos * theta^(-2j/dh), evaluated in fp64.
__device__ __forceinline__ float2 rope_angle(int pos, int j, int dh, float theta)
{
    const double freq = pow((double)theta, -2.0 * (double)j / (double)dh);
    double s, c;
    sincos((double)pos * freq, &s, &c);
    return make_float2((float)c, (float)s);
}

__global__ void rope_table_kernel(float2 *__restrict__ table, int max_pos, int dh, float theta)
{
    const int half = dh / 2;
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= max_pos * half) return;
    table[idx] = rope_angle(idx / half, idx % half, dh, theta);
}

// One workgroup per token row.  A thread rotates 8 pairs (j .. j+7, j+half ..)
// of one head of q or k: two 16-byte loads, two 16-byte stores.
__global__ __launch_bounds__(kThreads) void rope_kernel(uint16_t *__restrict__ qkv, const float2 *__restrict__ table,
                                                        int L, int H, int dh, float theta)
{
    const int r = blockIdx.x;
    const int pos = r % L;
    const int half = dh / 2, d = H * dh;
    const int per_head = half / 8;            // threads per head
    const int items = 2 * H * per_head;       // q heads then k heads
    uint16_t *row = qkv + (size_t)r * 3 * d;
    for (int it = threadIdx.x; it < items; it += kThreads) {
        const int hh = it / per_head;         // 0 .. 2H-1 (k heads follow q heads contiguously)
        const int j0 = (it % per_head) * 8;
        uint16_t *base = row + (size_t)hh * dh + j0;
        uint4 lo = *reinterpret_cast<uint4 *>(base);
        uint4 hi = *reinterpret_cast<uint4 *>(base + half);
        uint32_t *lw = reinterpret_cast<uint32_t *>(&lo), *hw = reinterpret_cast<uint32_t *>(&hi);
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            float a[2] = {bf16_lo(lw[p]), bf16_hi(lw[p])};
            float b[2] = {bf16_lo(hw[p]), bf16_hi(hw[p])};
            float oa[2], ob[2];
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const int j = j0 + 2 * p + e;
                const float2 cs = table ? table[(size_t)pos * half + j] : rope_angle(pos, j, dh, theta);
                oa[e] = a[e] * cs.x - b[e] * cs.y;
                ob[e] = a[e] * cs.y + b[e] * cs.x;
            }
            lw[p] = pack_bf16x2(oa[0], oa[1]);
            hw[p] = pack_bf16x2(ob[0], ob[1]);
        }
        *reinterpret_cast<uint4 *>(base) = lo;
        *reinterpret_cast<uint4 *>(base + half) = hi;
    }
}

}  // namespace

hipError_t launch_embed(hipStream_t stream, const int32_t *tokens, const int32_t *rows, const void *embed, float *x,
                        int M, int d, int vocab, int32_t *bad_token, const void *gain, void *h, int h_panel_rows,
                        float *ssq, int ssq_stride)
{
    if (gain && (!h || !ssq || ssq_stride < 1 || (h_panel_rows && (d % 32 || h_panel_rows < M)))) return hipErrorInvalidValue;
    hipLaunchKernelGGL(embed_kernel, dim3(M), dim3(kThreads), 0, stream, tokens, rows, (const uint16_t *)embed, x, d,
                       vocab, bad_token, (const uint16_t *)gain, (uint16_t *)h, h_panel_rows, ssq, ssq_stride);
    return hipGetLastError();
}

hipError_t launch_scatter_kv(hipStream_t stream, const void *src, void *dst, const int32_t *rows, int n_rows, int d)
{
    if (n_rows < 1) return hipSuccess;
    hipLaunchKernelGGL(scatter_kv_kernel, dim3(n_rows), dim3(kThreads), 0, stream, (const uint16_t *)src,
                       (uint16_t *)dst, rows, d);
    return hipGetLastError();
}

hipError_t launch_add_rmsnorm(hipStream_t stream, float *x, const float *partials, int n_partials, const void *gain,
                              void *h, int M, int d, float eps, int h_panel_rows)
{
    if (h_panel_rows && (d % 32 || h_panel_rows < M)) return hipErrorInvalidValue;
    hipLaunchKernelGGL(add_rmsnorm_kernel, dim3(M), dim3(kThreads), 0, stream, x, partials, n_partials,
                       (size_t)M * d, (const uint16_t *)gain, (uint16_t *)h, d, eps, h_panel_rows);
    return hipGetLastError();
}

hipError_t launch_rope_table(hipStream_t stream, float2 *table, int max_pos, int dh, float theta)
{
    const int n = max_pos * (dh / 2);
    hipLaunchKernelGGL(rope_table_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, table, max_pos, dh, theta);
    return hipGetLastError();
}

hipError_t launch_rope(hipStream_t stream, void *qkv, const float2 *table, int B, int L, int H, int dh, float theta)
{
    hipLaunchKernelGGL(rope_kernel, dim3(B * L), dim3(kThreads), 0, stream, (uint16_t *)qkv, table, L, H, dh, theta);
    return hipGetLastError();
}

}  // namespace dllm
