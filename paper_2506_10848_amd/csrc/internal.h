// Internal C++ interface between the C ABI layer and the kernel files.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/dllm.h"
#include "common.h"

namespace dllm {

// Window and rule of one sequence for one step, as the kernels want it.
struct SeqWindow {
    int lo, hi;  // inclusive span of positions the step decides on (hi < lo: nothing)
    int eval_hi; // masked positions in [lo, eval_hi] get a prediction and a confidence (>= hi)
    int stage;
    int top_k;
    float tau_min, tau_high;
    int conv_mode;
};
struct SelectArgs {
    SeqWindow w[DLLM_MAX_BATCH];
};
struct CommitOut {
    int capacity;
    int32_t *n_commit, *pos, *tok;
    float *conf;
    int32_t *e_cand, *first_masked, *n_masked_after;
};

hipError_t launch_row_phase(hipStream_t stream, const void *logits, int B, int L, int V, int mask_id,
                            const uint8_t *mask, const SelectArgs &args, int32_t *pred, float *conf);
hipError_t launch_seq_phase(hipStream_t stream, int B, int L, int32_t *tokens, uint8_t *mask, int32_t *prev_pred,
                            const int32_t *pred, const float *conf, const SelectArgs &args, const CommitOut &out);
// Row phase from the statistics that launch_gemm_rowstats left for rows first_row .. first_row + n_rows - 1.
hipError_t launch_rowstats_merge(hipStream_t stream, const float *stats, int parts, int n_rows, int first_row, int L,
                                 const uint8_t *mask, const SelectArgs &args, int32_t *pred, float *conf);

// ---- forward pass -------------------------------------------------------------
// rows (nullable): x[r] is the embedding of tokens[rows[r]] instead of tokens[r].  A token id outside
// [0, vocab) gives a row of zeros and sets *bad_token (device int32, nullable) to 1.
// gain (nullable): the kernel also leaves the operand of the first projection, h = bf16(x * gain) (row-major,
// or panel-major with h_panel_rows rows per panel), and ssq[r * ssq_stride] = sum of x[r]^2 (see RowScale).
hipError_t launch_embed(hipStream_t stream, const int32_t *tokens, const int32_t *rows, const void *embed, float *x,
                        int M, int d, int vocab, int32_t *bad_token, const void *gain = nullptr, void *h = nullptr,
                        int h_panel_rows = 0, float *ssq = nullptr, int ssq_stride = 0);
// dst[rows[r]][d .. 3d) = src[r][d .. 3d): the k and v thirds of recomputed rows go to their cache rows
hipError_t launch_scatter_kv(hipStream_t stream, const void *src, void *dst, const int32_t *rows, int n_rows, int d);
// h_panel_rows != 0: h is written panel-major (see GemmLayout) with that many rows per panel (>= M; d % 32 == 0)
hipError_t launch_add_rmsnorm(hipStream_t stream, float *x, const float *partials, int n_partials, const void *gain,
                              void *h, int M, int d, float eps, int h_panel_rows = 0);
hipError_t launch_rope_table(hipStream_t stream, float2 *table, int max_pos, int dh, float theta);
// table may be null: angles are then computed in the kernel (slow; test hook)
hipError_t launch_rope(hipStream_t stream, void *qkv, const float2 *table, int B, int L, int H, int dh, float theta);
// out_panel_rows != 0 (here and in launch_attention_rows): out is written panel-major (see GemmLayout)
hipError_t launch_attention(hipStream_t stream, const void *qkv, void *out, int B, int L, int H, int dh,
                            int out_panel_rows = 0);
// Queries of sequence b are the rows [first[b], first[b] + count[b]) of q (row stride 3d, q third);
// it attends to the Lk rows of kv that start at row b * Lk (k and v thirds); out rows as q rows.
struct SeqRows {
    int first[DLLM_MAX_BATCH], count[DLLM_MAX_BATCH];
};
hipError_t launch_attention_rows(hipStream_t stream, const void *q, const void *kv, void *out, int B, int Lk, int H,
                                 int dh, const SeqRows &rows, int out_panel_rows = 0);

// sink[workgroups * 256] floats; operands: n_operands pieces of 16 bytes (bf16 values); see probe.hip
hipError_t launch_mfma_rate(hipStream_t stream, const void *operands, int n_operands, float *sink, int workgroups,
                            int iters);

enum GemmEpilogue {
    kEpiBf16 = 0,     // C bf16 [M][N]
    kEpiSwiglu = 1,   // W = [gate | up] rows; C bf16 [M][N/2] = silu(gate) * up
    kEpiPartial = 2,  // C fp32 [splits][M][N], one slab per K split
};
// Layout of a product's operands and (SwiGLU only) of its output.  Row-major is the default.  Panel-major:
// a matrix X[rows][K] stored as [K / 32][panel_rows][32], i.e. panel p holds elements [32 p, 32 p + 32) of
// every row, rows contiguous (64 bytes each); the rows a product uses may be a range of the panel's rows
// (the operand pointer then points at the first of them inside panel 0).  A tile's K-stage is then one
// contiguous block in memory and every request to the L2 is a whole 128-byte line: measured on MI355X,
// the asynchronous tile copies reach 115 GB/s per CU from panel-major operands against 65 GB/s from
// row-major ones when the lines come from the L2, and 6.3 against 4.4 TB/s when they come from HBM.
// Only the asynchronous-copy kernel (K % 64 == 0, see gemm_async_copy_path) reads panel-major operands.
struct GemmLayout {
    int a_panel_rows = 0;  // 0: A row-major [M][K]; else rows per panel of a panel-major A
    int w_panel_rows = 0;  // 0: W row-major [N][K]; else rows per panel of a panel-major W (all N rows)
    int c_panel_rows = 0;  // kEpiSwiglu only: 0: output row-major [M][N/2]; else rows per panel of the output
};
// RMSNorm folded into the product that consumes the normalised rows.  The producer of the rows (the embedding
// kernel or the residual epilogue of the O / down projection) leaves bf16(x * gain) as the operand and, per
// row, `parts` partial sums of x^2 (ssq[row * stride + p]); the product then multiplies every output row by
// rsqrt(sum_p ssq / K + eps) in fp32 before its own epilogue, which is the same map as normalising first.
struct RowScale {
    const float *ssq = nullptr;  // null: rows are not scaled
    int parts = 0, stride = 0;
    float eps = 0.0f;
};
// What the residual product (launch_gemm_residual) updates and leaves for the next product:
//   x [M][N] fp32 += A W^T;  h = bf16(x * gain) row-major [M][N] or panel-major (h_panel_rows rows per panel);
//   ssq [M][ssq_stride]: per row, *ssq_parts partial sums of x^2.
// slabs: workspace for the fp32 partial tiles of split_limit K splits ([split_limit][M][N]); tickets: n_tickets
// zeroed int32 counters, one per output tile, left zeroed again (>= tiles of the narrowest plan).
struct ResidualOut {
    float *x = nullptr;
    const void *gain = nullptr;
    void *h = nullptr;
    int h_panel_rows = 0;
    float *ssq = nullptr;
    int ssq_stride = 0;
    float *slabs = nullptr;
    int *tickets = nullptr;
    int n_tickets = 0;
};
hipError_t launch_gemm_residual(hipStream_t stream, const void *A, const void *W, const ResidualOut &out, int M, int N,
                                int K, int split_limit, const GemmLayout &lay, int *ssq_parts);
int gemm_residual_max_parts(int N);
// Whether the product will run on the asynchronous-copy kernel (the one that takes panel-major operands).
bool gemm_async_copy_path(int epi, int M, int N, int K, int split_limit = 8);
// dst[K / 32][rows][32] (panel-major) = src[rows][K]; K % 32 == 0.
hipError_t launch_pack_panels(hipStream_t stream, const void *src, void *dst, size_t rows, int K);
// How many K splits launch_gemm will use for a kEpiPartial problem: between 1 and min(split_limit,
// kGemmMaxSplits).  The caller derives split_limit from the slab space it has and passes the same value
// to launch_gemm, so a plan never asks for more slabs than exist.
constexpr int kGemmMaxSplits = 8;
int gemm_num_splits(int M, int N, int K, int split_limit = kGemmMaxSplits);
// What launch_gemm (epi = a GemmEpilogue), launch_gemm_qkv_rope (epi = 3 for head_dim 64, 4 for 128) or
// launch_gemm_rowstats (epi = 5) will launch for a shape: tile, K depth of a stage, ring stages, wave grid,
// K splits, and whether it is the asynchronous-copy kernel (1) or the register-staged one (0).
struct GemmPlanInfo {
    int bm, bn, bk, stages, waves_m, waves_n, splits, async_copy;
};
GemmPlanInfo gemm_plan_info(int epi, int M, int N, int K, int split_limit = kGemmMaxSplits);
// Reads the DLLM_GEMM_* / DLLM_NO_FUSED_ROPE environment hooks again and forgets every cached plan
// (they are otherwise read once per process); for tests that switch kernels between calls.
void gemm_reload_env();
// QKV projection with the rotary embedding of the q and k thirds fused into the
// epilogue: C bf16 [M][3d] = A[M][d] * W[3d][d]^T, rows are positions row % L.
bool gemm_qkv_rope_supported(int M, int d, int dh);
// pos (nullable): position of every row; default row % L.  kv_dst / kv_rows (both or neither): the K and V
// thirds of output row r are written to row kv_rows[r] of kv_dst ([rows][3 d], e.g. a key/value cache) and
// only the Q third to row r of C.
hipError_t launch_gemm_qkv_rope(hipStream_t stream, const void *A, const void *W, void *C, int M, int d, int dh,
                                const float2 *table, int L, const int32_t *pos = nullptr,
                                const GemmLayout &lay = GemmLayout(), const RowScale &scale = RowScale(),
                                void *kv_dst = nullptr, const int32_t *kv_rows = nullptr);
// C = A[M][K] * W[N][K]^T.  For kEpiSwiglu N counts gate + up rows.
hipError_t launch_gemm(hipStream_t stream, GemmEpilogue epi, const void *A, const void *W, void *C, int M, int N,
                       int K, int split_limit = kGemmMaxSplits, const GemmLayout &lay = GemmLayout(),
                       const RowScale &scale = RowScale());
// The same product with the greedy decode fused in: no C; per row and per column slice (a wave's
// share of a tile, *parts of them) the maximum of the bf16-rounded values, the sum of
// exp(x - max) and the lowest column holding the maximum, column mask_id left out.
// stats: fp32/int32 planes [3][*parts][M]; *parts <= gemm_rowstats_max_parts(N).
size_t gemm_rowstats_max_parts(int N);
hipError_t launch_gemm_rowstats(hipStream_t stream, const void *A, const void *W, float *stats, int M, int N, int K,
                                int mask_id, int *parts, const GemmLayout &lay = GemmLayout(),
                                const RowScale &scale = RowScale());

}  // namespace dllm
