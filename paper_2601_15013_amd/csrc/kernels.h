// Internal launcher declarations (one per kernel family).  Host code; every launcher enqueues
// on `stream` and returns without synchronising.  Pointers are device pointers.
#pragma once
#include "common.h"

// The first bytes of every workspace: int32 words {status, n_compact, ...}.
#define RADIX_WS_HEADER_BYTES 256

size_t radix_index_ws_bytes(int B);

// ---- row operations (rowops.hip)
// dst[r, :] = src[idx[r], :]; row_bytes % 4 == 0.  idx == nullptr copies rows 1:1.  Rows r >= n_idx (n_idx < 0:
// none) take source row 0: the padding rows of a compact space rounded up to a bucket.
void launch_index_select_rows(const void* src, int n_src_rows, const int32_t* idx, int n_rows,
                              size_t row_bytes, void* dst, int32_t* status, hipStream_t stream, int n_idx = -1);
// Records RADIX_ERR_BAD_CU_SEQLENS in *status when cu is not 0 .. N non-decreasing with every
// sequence <= max_seqlen.  (Kernels that index through cu clamp what they read from it.)
void launch_validate_cu(const int32_t* cu, int B, int N, int max_seqlen, int32_t* status, hipStream_t stream);
// pos_full[i] = i - cu[seq(i)]
void launch_default_positions(const int32_t* cu, int B, int N, int32_t* pos_full, hipStream_t stream);
// ids_c[j] = tok[Ig[j]], pos_c[j] = pos[Ig[j]] for j < M_valid (Ig == nullptr: identity); rows M_valid <= j < M are
// padding: copies of token 0
void launch_compact_ids(const int32_t* tok, const int32_t* pos, const int32_t* Ig, int M, int M_valid, int N,
                        int vocab, int max_pos, int32_t* ids_c, int32_t* pos_c, int32_t* status,
                        hipStream_t stream);
// h[j, :] = (float) E[ids_c[j], :]
void launch_embed(const void* embed, int dtype, const int32_t* ids_c, int M, int d, float* h, hipStream_t stream);
// out[j, :] = h[j, :] * rsqrt(mean(h[j]^2) + eps) * g   (out in `out_dtype`: RADIX_F32 / RADIX_BF16 / RADIX_F16)
void launch_rmsnorm(const float* h, const float* g, int M, int d, float eps, void* out, int out_dtype,
                    hipStream_t stream);
// out[j, 0:d] = T(y), out[j, d:2d] = T(y - T(y)) with y the RMSNorm above: a hi/lo pair of 16-bit values
// (out_dtype RADIX_BF16 / RADIX_F16, d a multiple of 256).
int launch_rmsnorm_split(const float* h, const float* g, int M, int d, float eps, void* out, int out_dtype,
                         hipStream_t stream);
// In place on qkv[M, dq + 2 dkv]: per-head RMSNorm (optional) and RoPE of the q and k heads.
void launch_qknorm_rope(void* qkv, int dtype, int M, int n_q_heads, int n_kv_heads, int hd, int qk_norm,
                        const float* gq, const float* gk, float eps, const int32_t* pos_c,
                        const float* cos_tab, const float* sin_tab, hipStream_t stream);

// out[r, :] = (operand type) src[sel ? sel[r] : r, :] for r < n_rows; src is fp32 [n_src, d].  out_dtype RADIX_F32
// copies.  Entries of sel outside [0, n_src) are clamped and reported in *status.
void launch_rows_to_operand(const float* src, int n_src, const int32_t* sel, int n_rows, int d, void* out,
                            int out_dtype, int32_t* status, hipStream_t stream);

// dst[i] = (f16) src[i] for n bf16 values (weights handed over as bf16, multiplied as fp16)
void launch_bf16_to_f16(const bf16_t* src, f16_t* dst, size_t n, hipStream_t stream);

// ---- GEMMs: C[M, Nout] = A[M, K] * W[Nout, K]^T with an epilogue
enum GemmEpilogue {
    EPI_STORE = 0,     // C stored in the activation dtype
    EPI_RESIDUAL = 1,  // resid[M, Nout] (fp32) += C
    EPI_SWIGLU = 2,    // W holds gate/up interleaved in blocks of 32 rows; out[M, Nout/2] = silu(gate) * up
    EPI_QKV_ROPE = 3,  // EPI_STORE of the fused q|k|v row with per-head RMSNorm and RoPE applied to q and k heads
    EPI_STORE_F32 = 4, // C stored as fp32 (16-bit operand GEMMs only; the fp32 GEMM's EPI_STORE already is fp32)
    EPI_SWIGLU_SPLIT = 5  // EPI_SWIGLU with the result y written as a 16-bit (hi, lo) pair: out[M, 2 (Nout/2)] holds
                          // T(y) in columns [0, Nout/2) and T(y - T(y)) in columns [Nout/2, Nout)
};
// Extra inputs of EPI_QKV_ROPE (head_dim 128): gains and tables are device pointers.
struct QkvEpilogue {
    const float* gq;        // [128] q-norm gain
    const float* gk;        // [128] k-norm gain
    const float* cos_tab;   // [max_pos, 64]
    const float* sin_tab;   // [max_pos, 64]
    const int32_t* pos_c;   // [M] position id of every row
    int n_q_heads, n_kv_heads, qk_norm;
    float eps;
};
void launch_gemm_f32(const float* A, const float* W, int M, int Nout, int K, int epilogue, float* out_or_resid,
                     hipStream_t stream);
// 16-bit operands (op_dtype RADIX_BF16 or RADIX_F16), fp32 accumulate.  variant 0 = pick a tile shape.
// w_k: row length of W.  w_k == K is the plain product; w_k == K / 2 multiplies A = [hi | lo] against
// the weights repeated twice along k, i.e. C = (hi + lo) * W^T.
int launch_gemm_mfma(const void* A, const void* W, int M, int Nout, int K, int epilogue, void* out_or_resid,
                     int op_dtype, int variant, hipStream_t stream, const QkvEpilogue* qkv = nullptr, int w_k = 0);

// ---- causal varlen GQA attention on the full ragged layout.
// qkv[N, dq + 2 dkv] rows hold q | k | v of one token; out[N, dq].
void launch_attention_f32(const float* qkv, const int32_t* cu, int B, int N, int max_seqlen, int n_q_heads,
                          int n_kv_heads, int hd, float* out, hipStream_t stream);
// 16-bit operands (op_dtype RADIX_BF16 or RADIX_F16), head_dim 128.
// split_out != 0: out is [N, 2 dq] and a row holds T(o) in columns [0, dq) and T(o - T(o)) in columns [dq, 2 dq).
int launch_attention_mfma(const void* qkv, const int32_t* cu, int B, int N, int max_seqlen, int n_q_heads,
                          int n_kv_heads, int hd, void* out, int op_dtype, hipStream_t stream, int split_out = 0);
// The same attention with scatter and gather folded in: q | k | v rows are read from the COMPACT buffer
// qkv_c[n_compact, dq + 2 dkv] through I_scatter, only the representative positions of a sequence
// ([rep_start[b], len_b), see launch_rep_start) are computed, and their rows go straight to out_c[n_compact, dq].
int launch_attention_mfma_fused(const void* qkv_c, const int32_t* cu, const int32_t* I_scatter,
                                const int32_t* rep_start, int B, int N, int n_compact, int max_seqlen, int n_q_heads,
                                int n_kv_heads, int hd, void* out_c, int op_dtype, hipStream_t stream,
                                int split_out = 0);
// rep_start[b] = first position of sequence b whose token is its own representative (len_b if none).
void launch_rep_start(const int32_t* cu, const int32_t* I_scatter, const int32_t* I_gather, int B, int N,
                      int n_compact, int32_t* rep_start, hipStream_t stream);
