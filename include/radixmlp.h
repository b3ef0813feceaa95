/*
 * radixmlp.h - C ABI of the MI355X (gfx950) deduplicated-prefill library.
 *
 * The library implements the hot path of RadixMLP: a causal (Qwen3-style) decoder prefill
 * in which every position-wise operation runs on the unique prefix-trie rows ("compact
 * space", N' rows) and only causal attention runs on the full ragged layout (N rows)
 * (paper: Approach, "The RadixMLP Layout" and "Integration with Attention"; Algorithm 1).
 *
 * Conventions
 *   - Every array pointer is a DEVICE pointer unless its name ends in _host.
 *   - `stream` is a hipStream_t passed as void*; all device work is enqueued on it and,
 *     unless stated otherwise, the call returns without waiting for it.
 *   - The library never allocates caller-visible memory.  Scratch memory is a workspace
 *     the caller allocates (size from the *_workspace_bytes calls, 256-byte aligned) and
 *     passes to every call; calls that share a workspace must be ordered on one stream.
 *   - Every function returns 0 (RADIX_OK) or a negative radix_status.  Argument errors that
 *     are visible on the host are reported before anything is launched and nothing is
 *     written.  Errors in device-resident data (cu_seqlens not monotone, token id out of
 *     range) are recorded by the kernels in a status word inside the workspace; the
 *     kernels then leave outputs untouched or clamp the offending index, never read or
 *     write out of bounds, and the error is returned by radix_build_index itself when
 *     n_compact_host != NULL, else by radix_device_status.
 *   - Indices are 32-bit: N < 2^31.  Token ids and position ids must be >= 0.
 */
#ifndef RADIXMLP_H
#define RADIXMLP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum radix_status {
    RADIX_OK = 0,
    RADIX_ERR_NULL_POINTER = -1,
    RADIX_ERR_BAD_SIZE = -2,          /* negative B or N, N >= 2^31, n_compact > N, ... */
    RADIX_ERR_UNSUPPORTED = -3,       /* head_dim / dtype / shape the kernels do not cover */
    RADIX_ERR_WORKSPACE_TOO_SMALL = -4,
    RADIX_ERR_MISALIGNED = -5,        /* pointer not aligned as documented */
    RADIX_ERR_BAD_CU_SEQLENS = -6,    /* device data: cu_seqlens[0] != 0, decreasing, or last != N */
    RADIX_ERR_BAD_TOKEN = -7,         /* device data: token id < 0 or >= vocab, position id or row index out of range */
    RADIX_ERR_HIP = -8,               /* a HIP runtime call failed */
    RADIX_ERR_BAD_CONFIG = -9,        /* inconsistent model configuration */
    RADIX_ERR_STATIC_LIMIT = -10      /* radix_build_index_static: more sequences than its static scratch array holds */
} radix_status;

typedef enum radix_dtype { RADIX_F32 = 0, RADIX_BF16 = 1, RADIX_F16 = 2 } radix_dtype;

/* Shape of the decoder (paper: Background, Eqs. 1-2 and Eq. 5). */
typedef struct radix_model_config {
    int32_t n_layers;
    int32_t d;           /* hidden size */
    int32_t n_q_heads;   /* Hq */
    int32_t n_kv_heads;  /* Hkv, divides Hq */
    int32_t head_dim;    /* hd: even, <= 128; the bf16 path requires 128 */
    int32_t d_int;       /* SwiGLU intermediate size */
    int32_t vocab;
    int32_t max_pos;     /* RoPE table length; position ids must be < max_pos */
    int32_t qk_norm;     /* 1: per-head RMSNorm of q and k before RoPE (Qwen3) */
    int32_t dtype;       /* radix_dtype of the weights handed to radix_model_create: RADIX_F32 or RADIX_BF16 */
    int32_t compute_dtype; /* radix_dtype of activations and MFMA operands (accumulation is always fp32):
                              RADIX_F32 with fp32 weights; RADIX_BF16 or RADIX_F16 with bf16 weights.
                              RADIX_F16 converts the weights once at create time (exact for every bf16
                              value of magnitude >= 2^-17) and carries 11-bit instead of 8-bit
                              significands through the activations; activations must stay below 65504. */
    int32_t hilo_layers; /* Number of leading layers that carry every value they round to the operand type as a 16-bit
                            (hi, lo) pair: both RMSNorm outputs, the attention output and the SwiGLU output (their GEMMs
                            run over the doubled K against the weights read twice), and q, k, v (attention multiplies
                            K_hi Q_hi + K_hi Q_lo + K_lo Q_hi and adds V_hi and V_lo products).  About twice the
                            significand at those points for twice the GEMM work in those layers (bf16 weights only, d a
                            multiple of 256; q, k, v only when the fused q|k|v row is a multiple of 256 wide).  Rounding
                            errors of the first layer dominate the final error of deep models whose projections do not
                            attenuate (its outputs are the whole residual stream at that depth).
                            0: decided from the weights at create time: RADIX_HILO_AUTO_LAYERS layer(s) when
                               rms(Wq of layer 0) * sqrt(d) >= RADIX_HILO_AUTO_GAIN, else none;
                            k > 0: the first min(k, n_layers) layers;  -1: none. */
    int32_t fold_norms;  /* 1: fold every RMSNorm that sits between two 16-bit GEMMs into them (bf16 weights, d a multiple of
                            256, layers without (hi, lo) inputs): the O / down projection that last updates a residual row
                            also writes that row times the next norm's gain in the operand type and the row's sums of
                            squares, and the projection that follows scales its output rows by rsqrt(mean + eps); two
                            launches fewer per layer, same error.  0 (default): the norms run as kernels of their own,
                            which is what measures faster on an MI355X (the 16-bit write stays either way, the saved
                            fp32 read is worth less than what the longer GEMM epilogues and prologues cost: one
                            workgroup per compute unit, nothing overlaps them). */
    int32_t lm_head;     /* 0: no LM head (radix_lm_head returns RADIX_ERR_UNSUPPORTED); 1: head tied to the embedding
                            matrix; 2: separate matrix radix_weights.lm_head.  Non-zero makes radix_model_create
                            keep the head in the operand type (a converted copy of the embedding when that
                            differs from the weight type).  16-bit operand types need vocab % 128 == 0. */
    float eps;           /* RMSNorm epsilon (inside the square root) */
    float rope_base;
} radix_model_config;

/* The automatic setting of radix_model_config.hilo_layers. */
#define RADIX_HILO_AUTO_GAIN 0.85
#define RADIX_HILO_AUTO_LAYERS 1

/* Per-layer weights.  Matrices are [out, in] row-major as in y = W h (paper Eq. 5), stored
 * in config.dtype.  RMSNorm gains are always fp32.  All pointers are device pointers. */
typedef struct radix_layer_weights {
    const float* g1;   /* [d]      pre-attention norm gain */
    const void* wq;    /* [Hq*hd, d] */
    const void* wk;    /* [Hkv*hd, d] */
    const void* wv;    /* [Hkv*hd, d] */
    const float* gq;   /* [hd]     q-norm gain (ignored when qk_norm == 0) */
    const float* gk;   /* [hd]     k-norm gain */
    const void* wo;    /* [d, Hq*hd] */
    const float* g2;   /* [d]      post-attention norm gain */
    const void* wg;    /* [d_int, d] gate */
    const void* wu;    /* [d_int, d] up */
    const void* wd;    /* [d, d_int] down */
} radix_layer_weights;

typedef struct radix_weights {
    const void* embed;                       /* [vocab, d] in config.dtype (device) */
    const float* gf;                         /* [d] final norm gain (device) */
    const radix_layer_weights* layers_host;  /* HOST array of n_layers structs of device pointers */
    const void* lm_head;                     /* [vocab, d] in config.dtype (device); read only when config.lm_head == 2 */
} radix_weights;

typedef struct radix_model radix_model;      /* opaque */

#define RADIX_THRESHOLD_AUTO (-1.0f)
enum { RADIX_ATTN_AUTO = 0, RADIX_ATTN_THREE_KERNELS = 1, RADIX_ATTN_FUSED = 2 };

/* Options of the deduplicated forward (paper: Limitations, "Low-redundancy batches", and
 * the radix_mlp_threshold setting of the end-to-end experiments). */
typedef struct radix_fwd_opts {
    float threshold;      /* deduplicate iff n_compact < threshold * N; 1.0 = whenever anything is shared, 0.0 = never
                           * (the paper's radix_mlp_threshold).  Negative (RADIX_THRESHOLD_AUTO): the library decides, per
                           * batch: the position-wise work saved per layer, (N - N') * F / 1.1e15 s (F = projection + MLP flops of
                           * one row), against what deduplication adds - with the fused attention kernel about 15 % of
                           * the attention time, 0.15 * 2 * dq * N * (N / B) / 5e14 s; with the three-kernel attention the
                           * scatter of (N' + N) q|k|v rows at 5e12 bytes/s.  (Rates: what the kernels reach on an
                           * MI355X.)  E.g. 32 sequences of 1056 tokens: the 0.6B shape deduplicates below N'/N = 0.955 (fused
                           * attention) or 0.89 (three kernels), the 8B shape below 0.992 or 0.986.
                           * radix_dedup_decision evaluates the rule without running anything. */
    int32_t force_dedup;  /* 1: always take the deduplicated path, whatever the threshold says */
    int32_t attention_mode;  /* How scatter -> attention -> gather (Algorithm 1) is executed on the deduplicated path.
                              *  RADIX_ATTN_AUTO (0): the fused kernel where it applies (16-bit operand configurations,
                              *    compact q|k|v buffer below 4 GB), else the three kernels.
                              *  RADIX_ATTN_THREE_KERNELS (1): scatter of q|k|v to all N rows, attention on the full
                              *    ragged layout, gather of its output: the sequence as Algorithm 1 writes it.
                              *  RADIX_ATTN_FUSED (2): one attention kernel that reads q, k, v of the compact buffer
                              *    through I_scatter, computes only the representative positions (the rows the gather
                              *    would keep) and writes compact rows; same values bit for bit, no [N, .] copies.
                              *    RADIX_ERR_UNSUPPORTED with fp32 weights; falls back to the three kernels when the
                              *    compact q|k|v buffer reaches 4 GB.
                              *  Ignored when the threshold turns deduplication off. */
    int32_t pad_compact_to;  /* 0 or 1: off.  k > 1: the compact space is rounded up to a multiple of k rows (never
                              *    beyond N) with copies of the first representative, whose results are discarded
                              *    (paper: Implementation Details, performance padding): the position-wise kernels
                              *    then see one of few row counts, e.g. for graph capture per bucket.  Outputs are
                              *    unchanged bit for bit. */
} radix_fwd_opts;

/*
 * radix_model_create - validate the configuration, build library-owned device copies of the
 * weights in the layouts the kernels use (fused QKV matrix, gate/up interleaved, operand type) and the fp32
 * RoPE cos/sin tables (angle p * base^(-2i/hd) evaluated in double precision; element i is
 * paired with i + hd/2).  Synchronous.  The caller keeps ownership of the source weights and may
 * free them once the call returns.  On error *out is NULL.
 * radix_model_destroy frees everything the handle owns (NULL is accepted).
 */
int radix_model_create(const radix_model_config* config, const radix_weights* weights, radix_model** out);
int radix_model_destroy(radix_model* model);

/* Number of leading layers the model runs with (hi, lo) GEMM inputs: what radix_model_create resolved
 * radix_model_config.hilo_layers to (>= 0), or RADIX_ERR_NULL_POINTER. */
int radix_model_hilo_layers(const radix_model* model);

/* Bytes of workspace radix_build_index needs for batches of up to max_B sequences. */
int radix_index_workspace_bytes(int32_t max_B, size_t* bytes_out);

/* Bytes of workspace the forward calls need for up to max_N tokens in up to max_B sequences.
 * It is >= radix_index_workspace_bytes(max_B), so one buffer can serve both calls. */
int radix_workspace_bytes(const radix_model* model, int32_t max_N, int32_t max_B, size_t* bytes_out);

/*
 * radix_build_index - prefix-trie index maps of a ragged batch (paper: "Trie Construction",
 * "Gather and Scatter Kernels", appendix Algorithm 2 and its "Index semantics").
 *
 * Two original positions are the same trie node iff they sit at the same offset of their
 * sequences and the (token id, position id) pairs of their whole causal histories agree.
 *   I_gather[c]  (c < N') = smallest original position of compact node c; nodes are numbered
 *                           in order of first occurrence, so I_gather is strictly increasing.
 *   I_scatter[i] (i < N)  = compact node of original position i.
 * The result is the unique one the sequential algorithm produces; maps are never padded.
 *
 *   tok          int32[N]    token ids, >= 0
 *   pos          int32[N]    position ids, >= 0, or NULL for "offset inside the sequence"
 *   cu_seqlens   int32[B+1]  cu_seqlens[0] = 0, non-decreasing, cu_seqlens[B] = N; empty sequences allowed
 *   I_scatter    int32[N]    out
 *   I_gather     int32[N]    out; only the first N' entries are written
 *   n_compact_dev int32[1]   out (device), N'
 *   n_compact_host           HOST pointer or NULL.  If given, the call waits for the stream,
 *                            stores N' there and returns any device-data error.
 *   ws, ws_bytes             workspace of at least radix_index_workspace_bytes(B)
 * B = 0 or N = 0 is valid and yields N' = 0.
 */
int radix_build_index(const int32_t* tok, const int32_t* pos, const int32_t* cu_seqlens,
                      int32_t B, int32_t N, int32_t* I_scatter, int32_t* I_gather,
                      int32_t* n_compact_dev, int32_t* n_compact_host,
                      void* ws, size_t ws_bytes, void* stream);

/*
 * radix_build_index_static - radix_build_index for callers that cannot allocate device memory and so
 * have no workspace to pass: code that runs under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  Same arguments, same kernels and same results as radix_build_index, minus
 * ws / ws_bytes: the builder's state lives in a static device array inside the library
 * (about 160 KB, held by every GPU the library runs on until the process ends).  The call allocates
 * nothing and frees nothing.
 *   - At most RADIX_STATIC_INDEX_MAX_B sequences; more returns RADIX_ERR_STATIC_LIMIT before anything is
 *     launched.  N is not limited (the array holds per-sequence state only).
 *   - All calls on one GPU share that GPU's array: calls whose device work may overlap (different
 *     streams without ordering between them) race.  The array keeps the last call's contents; the
 *     kernels re-initialise every word they read, so nothing needs clearing between calls.
 *   - With n_compact_host == NULL nothing synchronises (graph capture: pass NULL).  Device-data errors are
 *     returned only when n_compact_host is given; there is no workspace for radix_device_status to
 *     read.  On a malformed cu_seqlens the maps are left untouched and n_compact_dev is set to 0.
 */
#define RADIX_STATIC_INDEX_MAX_B 4096
int radix_build_index_static(const int32_t* tok, const int32_t* pos, const int32_t* cu_seqlens,
                             int32_t B, int32_t N, int32_t* I_scatter, int32_t* I_gather,
                             int32_t* n_compact_dev, int32_t* n_compact_host, void* stream);

/*
 * radix_prefill_forward - deduplicated prefill (paper Algorithm 1 up to the final norm):
 * gathers token and position ids to compact space, runs embedding, RMSNorm, Q/K/V projection,
 * Q/K norm, RoPE, O projection, residual adds and the SwiGLU MLP on the n_compact unique rows,
 * scatters Q/K/V to the full ragged layout for causal varlen attention, gathers the attention
 * output back, and finally scatters the final-norm hidden state to all N rows.
 *
 *   tok, pos, cu_seqlens, B, N   as for radix_build_index (pos may be NULL); the forward calls take at most
 *                                65535 sequences per batch (B > 65535: RADIX_ERR_UNSUPPORTED)
 *   max_seqlen                   >= longest sequence (host value; sizes the attention grid)
 *   I_scatter, I_gather, n_compact   maps from radix_build_index for this batch (n_compact on the host)
 *   opts                         NULL = {RADIX_THRESHOLD_AUTO, force_dedup 0, RADIX_ATTN_AUTO, no padding}.  When the threshold says the
 *                                batch is not worth deduplicating the no-dedup path runs instead.
 *   out          float[N, d]     final-RMSNorm hidden state of every original token, ragged order
 *   ws, ws_bytes                 workspace of at least radix_workspace_bytes(model, N, B)
 * Asynchronous on `stream`.
 */
int radix_prefill_forward(const radix_model* model, const int32_t* tok, const int32_t* pos,
                          const int32_t* cu_seqlens, int32_t B, int32_t N, int32_t max_seqlen,
                          const int32_t* I_scatter, const int32_t* I_gather, int32_t n_compact,
                          const radix_fwd_opts* opts, float* out,
                          void* ws, size_t ws_bytes, void* stream);

/*
 * radix_dedup_decision - whether radix_prefill_forward would take the deduplicated path for a batch of B sequences,
 * N tokens and n_compact unique rows on a model of this configuration with these options (NULL = the defaults): the
 * rule documented at radix_fwd_opts.threshold (paper: Experiments, radix_mlp_threshold; Limitations,
 * "Low-redundancy batches").  Host arithmetic only: no GPU is touched, `config` is a host pointer, *dedup_out is set
 * to 1 or 0.  Errors: RADIX_ERR_NULL_POINTER, RADIX_ERR_BAD_SIZE (negative sizes, n_compact > N), the configuration
 * errors of radix_model_create, RADIX_ERR_BAD_CONFIG / RADIX_ERR_UNSUPPORTED for the attention mode as in
 * radix_prefill_forward.
 */
int radix_dedup_decision(const radix_model_config* config, int32_t B, int32_t N, int32_t n_compact,
                         const radix_fwd_opts* opts, int32_t* dedup_out);

/*
 * radix_prefill_forward_nodedup - the ordinary prefill over all N rows with the same kernels and
 * no gather/scatter: the baseline the paper's speedups are measured against (Experiments,
 * "RadixMLP disabled").  Arguments as above.
 */
int radix_prefill_forward_nodedup(const radix_model* model, const int32_t* tok, const int32_t* pos,
                                  const int32_t* cu_seqlens, int32_t B, int32_t N, int32_t max_seqlen,
                                  float* out, void* ws, size_t ws_bytes, void* stream);

/*
 * radix_lm_head - logits of selected rows (paper: Algorithm 1, output block, "logits = LMHead(h)"; a
 * bias-free linear map, tied to the embedding or a matrix of its own, see radix_model_config.lm_head).
 *   hidden    [n_src_rows, d] fp32: final-norm hidden states, i.e. what radix_prefill_forward wrote.
 *   rows      [n_rows] int32 row indices into hidden, or NULL for rows 0 .. n_rows-1 (n_rows <= n_src_rows).
 *             E.g. cu_seqlens[b+1]-1 for the last token of every sequence (a reranker's output), or
 *             I_gather for logits in compact space, which radix_index_select_rows with I_scatter then
 *             expands to all N rows (Algorithm 1: "y_c = LMHead(h), y = Scatter(y_c)").  An index outside
 *             [0, n_src_rows) is clamped and recorded as RADIX_ERR_BAD_TOKEN in the workspace status word.
 *   logits    [n_rows, vocab] fp32, 16-byte aligned.
 *   ws        at least radix_lm_head_workspace_bytes(model, n_rows) bytes, 256-byte aligned; may be the
 *             forward's workspace when that is large enough (the status word is shared, the rest reused).
 * Rows are converted to the operand type (one rounding for 16-bit operands), multiplied with fp32
 * accumulation in a fixed order (a row's logits do not depend on which other rows are selected).
 * Asynchronous on `stream`.
 */
int radix_lm_head_workspace_bytes(const radix_model* model, int32_t max_rows, size_t* bytes_out);
int radix_lm_head(const radix_model* model, const float* hidden, int32_t n_src_rows, const int32_t* rows,
                  int32_t n_rows, float* logits, void* ws, size_t ws_bytes, void* stream);

/*
 * radix_index_select_rows - the gather/scatter operator itself (paper: Implementation Details,
 * Gather(t, I)[j] = t[I[j]] and Scatter(t, I)[i] = t[I[i]]; both are row index-selects):
 * dst[r, :] = src[idx[r], :] for r < n_rows.  row_bytes must be a multiple of 4; rows are
 * contiguous.  Indices must lie in [0, n_src_rows); an index outside is clamped and recorded
 * as RADIX_ERR_BAD_TOKEN in *status_dev when status_dev != NULL.
 */
int radix_index_select_rows(const void* src, int32_t n_src_rows, const int32_t* idx, int32_t n_rows,
                            size_t row_bytes, void* dst, int32_t* status_dev, void* stream);

/* Waits for `stream` and returns the device-data status recorded in the workspace by the most
 * recent radix_build_index / radix_prefill_forward* call that used it (each call starts by
 * clearing the status word; RADIX_OK if nothing was recorded). */
int radix_device_status(void* ws, size_t ws_bytes, void* stream);

/* Static description of a radix_status value. */
const char* radix_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* RADIXMLP_H */
