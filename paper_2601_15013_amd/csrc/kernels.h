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
    EPI_QKV_ROPE_SPLIT = 7, // EPI_QKV_ROPE with every q | k | v value y written as a 16-bit (hi, lo) pair: out[M, 2 Nout]
                            // holds T(y) in columns [0, Nout) and T(y - T(y)) in columns [Nout, 2 Nout)
    EPI_RESIDUAL_NORM = 6, // EPI_RESIDUAL that also prepares the RMSNorm of the updated rows (NormFusion, producer side)
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
// RMSNorm folded into the GEMMs on either side of it (paper: Algorithm 1, the "LayerNorm" lines in front of
// "QKVProj" and "MLP"; read as RMSNorm).  y = x * rsqrt(mean(x^2) + eps) * g feeds a projection, and the row
// scalar rsqrt(..) commutes with it, so:
//   producer (EPI_RESIDUAL_NORM, the O / down projection that last updates the residual row x): besides
//     resid += C it writes a16[m, :] = T(x[m, :] * gain[:]), the un-normalised operand of the next projection, and
//     ss_out[m, s] = sum of x[m, c]^2 over the 128 columns c of slot s, summed in a fixed in-lane order that does
//     not depend on M, on the tile shape or on where the row sits (every tile shape that may run this epilogue
//     gives a wavefront exactly 128 columns);
//   consumer (any 16-bit epilogue, ss_in != nullptr): row m of the product is multiplied by
//     rsqrt(sum_s ss_in[m, s] * inv_d + eps) before the epilogue proper.
struct NormFusion {
    void* a16;            // producer: [M, Nout] in the operand type
    const float* gain;    // producer: [Nout] gain of the norm that follows
    float* ss_out;        // producer: [M, Nout / 128]
    const float* ss_in;   // consumer: [M, n_slots_in] or nullptr
    int n_slots_in;       // consumer: even
    float inv_d, eps;     // consumer: 1 / (normalised width), epsilon inside the square root
};

// Optional row map of the A operand: row m of the product reads row rows[m] of A[n_src, K] for m < n_valid and row 0
// beyond (Gather(t, I)[j] = t[I[j]] applied while loading); bad entries are clamped and recorded in *status.
// Needs n_src * K * 2 < 2^32.
struct ARowMap {
    const int32_t* rows;
    int n_valid, n_src;
    int32_t* status;
};
void launch_gemm_f32(const float* A, const float* W, int M, int Nout, int K, int epilogue, float* out_or_resid,
                     hipStream_t stream);
// Tile numbering of the MFMA GEMM: which output tile (row tile tm, column tile tn) the workgroup with id `bid`
// computes, for a launch of tiles_m * tiles_n workgroups.  Workgroup ids go round-robin to the 8 XCDs (own L2
// each): XCD x runs ids x, x + 8, ... in order.  Row tiles are grouped in bands of `band` that sweep the column
// (weight) tiles.  While there are 8 whole bands left, each XCD takes one of them and all eight sweep the columns
// in step, so that a weight strip is asked for by all XCDs at about the same time and has to stay in the
// memory-side cache only that long; every other sweep runs backwards, starting on the weight strips used last.
// The rows left over (fewer than 8 bands) are split evenly: each XCD gets a contiguous run of their tiles in band
// order.  Every tile is computed by exactly one workgroup (tested on the host).
struct GemmTile { int tm, tn; };
__host__ __device__ inline GemmTile gemm_tile_of(int bid, int tiles_m, int tiles_n, int band) {
    const int x = bid % 8, q = bid / 8;
    const int band_tiles = band * tiles_n;
    const int S = tiles_m / (8 * band);                  // sweeps with one whole band per XCD
    const int P1 = S * band_tiles;
    int row0, band_rows, in_band, tn;
    if (q < P1) {
        const int sidx = q / band_tiles;
        in_band = q - sidx * band_tiles;
        row0 = (sidx * 8 + x) * band;
        band_rows = band;
        tn = in_band / band_rows;
        if (sidx & 1) tn = tiles_n - 1 - tn;
    } else {
        const int R = tiles_m - S * 8 * band;
        const int nblk = R * tiles_n;
        const int per = nblk / 8, rem = nblk % 8;       // XCD x gets `per` (+1 if x < rem) blocks
        const int pid = x * per + (x < rem ? x : rem) + (q - P1);
        const int b = pid / band_tiles;
        band_rows = (R - b * band) < band ? (R - b * band) : band;
        in_band = pid - b * band_tiles;
        row0 = S * 8 * band + b * band;
        tn = in_band / band_rows;
    }
    GemmTile t;
    t.tm = row0 + in_band % band_rows;
    t.tn = tn;
    return t;
}
// Row tiles per band.  The 32 workgroups an XCD runs at a time cover band x (32 / band) tiles, i.e.
// band + 32 / band operand strips stream through its L2: 12 for a band of 4 or 8, 18 for 2.  The activation strips
// of a band are read again for every group of column tiles, and what serves those re-reads is the 256 MB
// memory-side cache shared by all XCDs: the eight bands in flight must leave room in it for the weights, so long
// rows (large K) take a narrower band.  Measured on MI355X, us per launch with bands of 8 / 4 / 2 / 1:
// M 45120, N 4096, K 12288: 4210 / 4168 / 4134 / 4109; N 24576, K 4096: 7109 / 7025 / 7105 / 7821;
// N 6144, K 4096: 1827 / 1841 / 1840 / 1929.
inline int gemm_band_rows(int bm, int K, int elem_bytes, int tiles_n) {
    int band = 8;
    while (band > 1 && 8.0 * band * bm * (double)K * elem_bytes > 64.0 * 1024 * 1024) band /= 2;
    if (band == 1 && tiles_n > 16) band = 2;          // one row of many column tiles: 33 strips per group
    return band;
}

// 16-bit operands (op_dtype RADIX_BF16 or RADIX_F16), fp32 accumulate.  variant 0 = pick a tile shape.
// w_k: row length of W.  w_k == K is the plain product; w_k == K / 2 multiplies A = [hi | lo] against
// the weights repeated twice along k, i.e. C = (hi + lo) * W^T.
int launch_gemm_mfma(const void* A, const void* W, int M, int Nout, int K, int epilogue, void* out_or_resid,
                     int op_dtype, int variant, hipStream_t stream, const QkvEpilogue* qkv = nullptr, int w_k = 0,
                     const ARowMap* a_rows = nullptr, const NormFusion* norm = nullptr);

// ---- causal varlen GQA attention on the full ragged layout.
// qkv[N, dq + 2 dkv] rows hold q | k | v of one token; out[N, dq].
void launch_attention_f32(const float* qkv, const int32_t* cu, int B, int N, int max_seqlen, int n_q_heads,
                          int n_kv_heads, int hd, float* out, hipStream_t stream);
// 16-bit operands (op_dtype RADIX_BF16 or RADIX_F16), head_dim 128.
// split_out != 0: out is [N, 2 dq] and a row holds T(o) in columns [0, dq) and T(o - T(o)) in columns [dq, 2 dq).
// split_in != 0: qkv is [N, 2 (dq + 2 dkv)], a row holds q | k | v (hi parts) and then q | k | v (lo parts).
int launch_attention_mfma(const void* qkv, const int32_t* cu, int B, int N, int max_seqlen, int n_q_heads,
                          int n_kv_heads, int hd, void* out, int op_dtype, hipStream_t stream, int split_out = 0,
                          int split_in = 0);
// The same attention with scatter and gather folded in: q | k | v rows are read from the COMPACT buffer
// qkv_c[n_compact, dq + 2 dkv] through I_scatter, only the representative positions of a sequence are computed,
// and their rows go straight to out_c[n_compact, dq] (split_out: [n_compact, 2 dq], hi | lo).  The work list
// comes from launch_attn_plan (same cu / I_scatter / n_q_heads / n_kv_heads).
int launch_attention_mfma_fused(const void* qkv_c, const int32_t* cu, const int32_t* I_scatter,
                                const int32_t* plan, int B, int N, int n_compact, int n_q_heads,
                                int n_kv_heads, int hd, void* out_c, int op_dtype, hipStream_t stream,
                                int split_out = 0, int split_in = 0);

// Work list of the fused attention kernel, built once per forward.  The representative positions of sequence
// b are its tail [first_b, len_b) (first_b: the first position whose token is its own representative); they are
// cut into blocks of 32 query rows.  A workgroup serves `slots` blocks (slots = 4 / min(group, 4) wavefronts per
// query head): `slots` consecutive blocks of one sequence where a sequence has that many left, else the leftover
// blocks of consecutive sequences packed together, which then share the K/V tiles of their common prefix.
// Layout of plan[] (int32): [0] number of items, [1] number of single-sequence items; per-sequence scratch; per
// item: t_shared (K/V tiles of 64 keys that all slots walk together; INT_MAX: all of them), seq[4], q[4]
// (sequence and first query position of every slot, seq = -1: empty slot).
struct AttnPlanLayout {
    size_t first, lcp, nfull, nrem, t_shared, seq, q, total;   // offsets in int32 words
    int max_items;
};
static inline AttnPlanLayout attn_plan_layout(size_t N, size_t B) {
    AttnPlanLayout L;
    L.max_items = (int)(N / 32 + B + 1);
    size_t off = 4;
    L.first = off; off += B;
    L.lcp = off; off += B;
    L.nfull = off; off += B;
    L.nrem = off; off += B;
    L.t_shared = off; off += (size_t)L.max_items;
    L.seq = off; off += 4 * (size_t)L.max_items;
    L.q = off; off += 4 * (size_t)L.max_items;
    L.total = off;
    return L;
}
void launch_attn_plan(const int32_t* cu, const int32_t* I_scatter, const int32_t* I_gather, int B, int N,
                      int n_compact, int n_q_heads, int n_kv_heads, int32_t* plan, hipStream_t stream);
