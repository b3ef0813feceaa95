// Model handle (library-owned weight copies + RoPE tables), workspace layout and the host-side
// launch sequence of the deduplicated / no-dedup prefill (paper: Algorithm 1).
#include <math.h>
#include <new>
#include <vector>

#include "common.h"
#include "kernels.h"
#include "radixmlp_bench.h"

struct radix_layer_dev {
    const float *g1, *g2, *gq, *gk;
    const void *wqkv;   // [dq + 2 dkv, d]  rows: q heads, k heads, v heads
    const void *wo;     // [d, dq]
    const void *wgu;    // [2 d_int, d]     gate/up interleaved in blocks of 32 rows
    const void *wd;     // [d, d_int]
};

struct radix_model {
    radix_model_config cfg;
    int hilo_layers = 0;           // resolved count of leading layers that carry GEMM inputs as (hi, lo) pairs
    char* blob = nullptr;          // one device allocation holding everything below
    const void* embed = nullptr;
    const void* lm_head = nullptr;  // [vocab, d] in the operand type (may alias embed), or null
    const float* gf = nullptr;
    const float* cos_tab = nullptr;
    const float* sin_tab = nullptr;
    std::vector<radix_layer_dev> layers;
};

namespace {

// ---- optional per-kernel timing with HIP events on the caller's stream (used by the benchmark
// to measure a kernel's average launch duration inside the timed region)
struct KernelTimer {
    uint32_t mask = 0;
    uint32_t stride = 1;                                   // bracket every stride-th launch of a category
    size_t seen[RADIX_TIMING_CATEGORIES] = {};
    std::vector<std::pair<hipEvent_t, hipEvent_t>> pool[RADIX_TIMING_CATEGORIES];
    size_t used[RADIX_TIMING_CATEGORIES] = {};
    int begin(int cat, hipStream_t s) {
        if (!(mask >> cat & 1u)) return -1;
        if (seen[cat]++ % stride != 0) return -1;
        if (used[cat] == pool[cat].size()) {
            hipEvent_t a, b;
            if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) return -1;
            pool[cat].push_back({a, b});
        }
        (void)hipEventRecord(pool[cat][used[cat]].first, s);
        return (int)used[cat];
    }
    void end(int cat, int slot, hipStream_t s) {
        if (slot < 0) return;
        (void)hipEventRecord(pool[cat][slot].second, s);
        used[cat] = (size_t)slot + 1;
    }
};
KernelTimer g_timer;

struct TimedScope {
    int cat, slot;
    hipStream_t s;
    TimedScope(int c, hipStream_t st) : cat(c), slot(g_timer.begin(c, st)), s(st) {}
    ~TimedScope() { g_timer.end(cat, slot, s); }
};

__global__ void interleave_gate_up_kernel(const uint4* __restrict__ wg, const uint4* __restrict__ wu, int d_int,
                                          int row_vecs, uint4* __restrict__ dst) {
    const int R = blockIdx.x;                  // destination row in [0, 2 d_int)
    const int t = R >> 6, w = R & 63;
    const uint4* src = (w < 32 ? wg : wu) + (size_t)(32 * t + (w & 31)) * row_vecs;
    uint4* d = dst + (size_t)R * row_vecs;
    for (int c = threadIdx.x; c < row_vecs; c += blockDim.x) d[c] = src[c];
}

__global__ void clear_status_kernel(int32_t* hdr) { hdr[0] = 0; }

// Sum of squares of n 16-bit weights, one workgroup, fixed order (the result decides a setting, so it must
// not depend on scheduling): thread t sums elements t, t + 1024, ...; then wavefront and workgroup reductions.
__global__ __launch_bounds__(1024) void sum_squares_bf16_kernel(const bf16_t* __restrict__ w, size_t n,
                                                                float* __restrict__ out) {
    __shared__ float part[16];
    float ss = 0.f;
    for (size_t i = threadIdx.x; i < n; i += 1024) { const float v = (float)w[i]; ss += v * v; }
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
    __syncthreads();
    if (threadIdx.x == 0) {
        float t = 0.f;
        for (int k = 0; k < 16; ++k) t += part[k];
        *out = t;
    }
}

size_t esize(int dtype) { return dtype == RADIX_F32 ? 4 : 2; }

struct WsLayout {
    size_t pos_full, ids_c, pos_c, plan, h, ss, a, qkv, qkv_full, attn_full, attn_c, mlp, ynorm, total;
};

WsLayout ws_layout(const radix_model_config& c, int hilo_layers, size_t N, size_t B) {
    const size_t es = esize(c.compute_dtype);
    const size_t dq = (size_t)c.n_q_heads * c.head_dim, dkv = (size_t)c.n_kv_heads * c.head_dim;
    const size_t row = dq + 2 * dkv;
    const size_t M = N;                       // worst case: nothing is shared
    size_t off = radix_index_ws_bytes((int)B);
    auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes ? bytes : 1, 256); return o; };
    WsLayout L;
    L.pos_full = take(N * 4);
    L.ids_c = take(M * 4);
    L.pos_c = take(M * 4);
    L.plan = take(attn_plan_layout(N, B).total * 4);
    L.h = take(M * c.d * 4);
    L.ss = take(M * ((size_t)c.d / 128 + 1) * 4);      // per-row sums of squares in 128-column slots (RMSNorm folded into the GEMMs)
    const size_t w2 = hilo_layers > 0 ? 2 : 1;     // (hi, lo) rows are twice as wide
    L.a = take(M * c.d * es * w2);
    L.qkv = take(M * row * es * w2);
    L.qkv_full = take(N * row * es * w2);
    L.attn_full = take(N * dq * es * w2);
    L.attn_c = take(M * dq * es * w2);
    L.mlp = take(M * (size_t)c.d_int * es * w2);
    L.ynorm = take(M * c.d * 4);
    L.total = off;
    return L;
}

int check_config(const radix_model_config& c) {
    if (c.n_layers <= 0 || c.d <= 0 || c.n_q_heads <= 0 || c.n_kv_heads <= 0 || c.head_dim <= 0 || c.d_int <= 0 ||
        c.vocab <= 0 || c.max_pos <= 0)
        return RADIX_ERR_BAD_CONFIG;
    if (c.n_q_heads % c.n_kv_heads != 0) return RADIX_ERR_BAD_CONFIG;
    if (!(c.eps >= 0.f) || !(c.rope_base > 0.f)) return RADIX_ERR_BAD_CONFIG;
    if (c.dtype != RADIX_F32 && c.dtype != RADIX_BF16) return RADIX_ERR_UNSUPPORTED;
    if (c.dtype == RADIX_F32 && c.compute_dtype != RADIX_F32) return RADIX_ERR_UNSUPPORTED;
    if (c.dtype == RADIX_BF16 && c.compute_dtype != RADIX_BF16 && c.compute_dtype != RADIX_F16) return RADIX_ERR_UNSUPPORTED;
    if (c.head_dim % 2 != 0 || c.head_dim > 128) return RADIX_ERR_UNSUPPORTED;
    if (c.d_int % 32 != 0) return RADIX_ERR_UNSUPPORTED;       // gate/up interleave granularity
    if (c.d % 4 != 0 || c.head_dim % 4 != 0) return RADIX_ERR_UNSUPPORTED;   // 16-byte rows
    if (c.hilo_layers < -1) return RADIX_ERR_BAD_CONFIG;
    if (c.fold_norms != 0 && c.fold_norms != 1) return RADIX_ERR_BAD_CONFIG;
    if (c.lm_head < 0 || c.lm_head > 2) return RADIX_ERR_BAD_CONFIG;
    if (c.lm_head && c.dtype == RADIX_BF16 && (c.vocab % 128 != 0)) return RADIX_ERR_UNSUPPORTED;
    if (c.hilo_layers > 0 && (c.dtype != RADIX_BF16 || c.d % 256 != 0)) return RADIX_ERR_UNSUPPORTED;
    if (c.dtype == RADIX_BF16) {
        // shapes the MFMA kernels cover: head_dim 128, every GEMM K a multiple of 32 and every
        // GEMM output width a multiple of 128
        const int dq = c.n_q_heads * c.head_dim, dkv = c.n_kv_heads * c.head_dim;
        if (c.head_dim != 128) return RADIX_ERR_UNSUPPORTED;
        if (c.d % 128 != 0 || c.d_int % 64 != 0 || (dq + 2 * dkv) % 128 != 0) return RADIX_ERR_UNSUPPORTED;
    }
    return RADIX_OK;
}

}  // namespace

extern "C" int radix_model_create(const radix_model_config* config, const radix_weights* weights, radix_model** out) {
    if (!out) return RADIX_ERR_NULL_POINTER;
    *out = nullptr;
    if (!config || !weights) return RADIX_ERR_NULL_POINTER;
    const radix_model_config c = *config;
    int rc = check_config(c);
    if (rc != RADIX_OK) return rc;
    if (!weights->embed || !weights->gf || !weights->layers_host) return RADIX_ERR_NULL_POINTER;
    if (c.lm_head == 2 && !weights->lm_head) return RADIX_ERR_NULL_POINTER;
    for (int l = 0; l < c.n_layers; ++l) {
        const radix_layer_weights& w = weights->layers_host[l];
        if (!w.g1 || !w.wq || !w.wk || !w.wv || !w.wo || !w.g2 || !w.wg || !w.wu || !w.wd) return RADIX_ERR_NULL_POINTER;
        if (c.qk_norm && (!w.gq || !w.gk)) return RADIX_ERR_NULL_POINTER;
    }
    const size_t es = esize(c.dtype);       // weights are stored at their own width; 16-bit operand types share it
    const size_t d = c.d, hd = c.head_dim, dq = (size_t)c.n_q_heads * hd, dkv = (size_t)c.n_kv_heads * hd;
    const size_t di = c.d_int, half = hd / 2;

    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes, 256); return o; };
    const size_t o_embed = take((size_t)c.vocab * d * es), o_gf = take(d * 4);
    // the head needs a copy of its own unless it is the embedding matrix and that already has the operand type
    const bool head_converted = c.dtype == RADIX_BF16 && c.compute_dtype == RADIX_F16;
    const bool head_copy = c.lm_head == 2 || (c.lm_head == 1 && head_converted);
    const size_t o_head = head_copy ? take((size_t)c.vocab * d * es) : 0;
    const size_t o_cos = take((size_t)c.max_pos * half * 4), o_sin = take((size_t)c.max_pos * half * 4);
    struct LO { size_t g1, g2, gq, gk, wqkv, wo, wgu, wd; };
    std::vector<LO> lo(c.n_layers);
    for (int l = 0; l < c.n_layers; ++l) {
        lo[l].g1 = take(d * 4); lo[l].g2 = take(d * 4); lo[l].gq = take(hd * 4); lo[l].gk = take(hd * 4);
        lo[l].wqkv = take((dq + 2 * dkv) * d * es);
        lo[l].wo = take(d * dq * es);
        lo[l].wgu = take(2 * di * d * es);
        lo[l].wd = take(d * di * es);
    }
    radix_model* m = new (std::nothrow) radix_model();
    if (!m) return RADIX_ERR_HIP;
    m->cfg = c;
    if (hipMalloc((void**)&m->blob, off) != hipSuccess) { delete m; return RADIX_ERR_HIP; }
    char* b = m->blob;
    bool ok = true;
    auto d2d = [&](size_t dst, const void* src, size_t bytes) {
        if (ok && hipMemcpyAsync(b + dst, src, bytes, hipMemcpyDeviceToDevice, 0) != hipSuccess) ok = false;
    };
    d2d(o_embed, weights->embed, (size_t)c.vocab * d * es);
    d2d(o_gf, weights->gf, d * 4);
    {
        std::vector<float> ct((size_t)c.max_pos * half), st((size_t)c.max_pos * half);
        for (size_t i = 0; i < half; ++i) {
            const double theta = pow((double)c.rope_base, -2.0 * (double)i / (double)hd);
            for (size_t p = 0; p < (size_t)c.max_pos; ++p) {
                const double ang = (double)p * theta;
                ct[p * half + i] = (float)cos(ang);
                st[p * half + i] = (float)sin(ang);
            }
        }
        if (hipMemcpy(b + o_cos, ct.data(), ct.size() * 4, hipMemcpyHostToDevice) != hipSuccess) ok = false;
        if (hipMemcpy(b + o_sin, st.data(), st.size() * 4, hipMemcpyHostToDevice) != hipSuccess) ok = false;
    }
    m->embed = b + o_embed;
    if (c.lm_head) {
        if (head_copy) {
            d2d(o_head, c.lm_head == 2 ? weights->lm_head : weights->embed, (size_t)c.vocab * d * es);
            if (head_converted)
                launch_bf16_to_f16((const bf16_t*)(b + o_head), (f16_t*)(b + o_head), (size_t)c.vocab * d, 0);
            m->lm_head = b + o_head;
        } else {
            m->lm_head = b + o_embed;
        }
    }
    m->gf = (const float*)(b + o_gf);
    m->cos_tab = (const float*)(b + o_cos);
    m->sin_tab = (const float*)(b + o_sin);
    m->layers.resize(c.n_layers);
    const int row_vecs = (int)(d * es / 16);
    for (int l = 0; l < c.n_layers && ok; ++l) {
        const radix_layer_weights& w = weights->layers_host[l];
        d2d(lo[l].g1, w.g1, d * 4);
        d2d(lo[l].g2, w.g2, d * 4);
        if (c.qk_norm) { d2d(lo[l].gq, w.gq, hd * 4); d2d(lo[l].gk, w.gk, hd * 4); }
        d2d(lo[l].wqkv, w.wq, dq * d * es);
        d2d(lo[l].wqkv + dq * d * es, w.wk, dkv * d * es);
        d2d(lo[l].wqkv + (dq + dkv) * d * es, w.wv, dkv * d * es);
        d2d(lo[l].wo, w.wo, d * dq * es);
        d2d(lo[l].wd, w.wd, d * di * es);
        if ((((uintptr_t)w.wg | (uintptr_t)w.wu) & 15) != 0) { ok = false; rc = RADIX_ERR_MISALIGNED; break; }
        hipLaunchKernelGGL(interleave_gate_up_kernel, dim3((unsigned)(2 * di)), dim3(256), 0, 0, (const uint4*)w.wg,
                           (const uint4*)w.wu, (int)di, row_vecs, (uint4*)(b + lo[l].wgu));
        if (c.dtype == RADIX_BF16 && c.compute_dtype == RADIX_F16) {
            // multiply in fp16: every bf16 weight of magnitude >= 2^-17 is represented exactly
            const size_t first = lo[l].wqkv, last = lo[l].wd + d * di * es;
            launch_bf16_to_f16((const bf16_t*)(b + first), (f16_t*)(b + first), (last - first) / 2, 0);
        }
        radix_layer_dev& L = m->layers[l];
        L.g1 = (const float*)(b + lo[l].g1); L.g2 = (const float*)(b + lo[l].g2);
        L.gq = (const float*)(b + lo[l].gq); L.gk = (const float*)(b + lo[l].gk);
        L.wqkv = b + lo[l].wqkv; L.wo = b + lo[l].wo; L.wgu = b + lo[l].wgu; L.wd = b + lo[l].wd;
    }
    // Leading layers with (hi, lo) GEMM inputs.  0 = decide from the weights: a projection with weights of
    // root-mean-square s and fan-in d multiplies a perturbation of its (normalised) input by about s sqrt(d).
    // Where that gain reaches 1, rounding errors made in the first layers - whose outputs ARE the residual stream
    // at that depth - are carried undiminished through all later layers, and two layers of doubled significand
    // remove most of the final error; below 1 they fade and the plain path is already an order of magnitude
    // inside the tolerance.
    m->hilo_layers = c.hilo_layers < 0 ? 0 : (c.hilo_layers < c.n_layers ? c.hilo_layers : c.n_layers);
    if (ok && c.hilo_layers == 0 && c.dtype == RADIX_BF16 && c.d % 256 == 0) {
        float* ss_dev = nullptr;
        float ss = 0.f;
        if (hipMalloc((void**)&ss_dev, sizeof(float)) != hipSuccess) ok = false;
        if (ok) {
            hipLaunchKernelGGL(sum_squares_bf16_kernel, dim3(1), dim3(1024), 0, 0,
                               (const bf16_t*)weights->layers_host[0].wq, dq * d, ss_dev);
            if (hipMemcpy(&ss, ss_dev, sizeof(float), hipMemcpyDeviceToHost) != hipSuccess) ok = false;
            (void)hipFree(ss_dev);
        }
        const double gain = sqrt((double)ss / (double)(dq * d)) * sqrt((double)d);
        if (ok && gain >= RADIX_HILO_AUTO_GAIN) m->hilo_layers = c.n_layers < RADIX_HILO_AUTO_LAYERS ? c.n_layers : RADIX_HILO_AUTO_LAYERS;
    }
    if (ok && hipDeviceSynchronize() != hipSuccess) ok = false;
    if (ok && hipGetLastError() != hipSuccess) ok = false;
    if (!ok) {
        (void)hipFree(m->blob);
        delete m;
        return rc != RADIX_OK ? rc : RADIX_ERR_HIP;
    }
    *out = m;
    return RADIX_OK;
}

extern "C" int radix_model_destroy(radix_model* model) {
    if (!model) return RADIX_OK;
    hipError_t e = hipFree(model->blob);
    delete model;
    return e == hipSuccess ? RADIX_OK : RADIX_ERR_HIP;
}

extern "C" int radix_model_hilo_layers(const radix_model* model) {
    return model ? model->hilo_layers : (int)RADIX_ERR_NULL_POINTER;
}

extern "C" int radix_workspace_bytes(const radix_model* model, int32_t max_N, int32_t max_B, size_t* bytes_out) {
    if (!model || !bytes_out) return RADIX_ERR_NULL_POINTER;
    if (max_N < 0 || max_B < 0) return RADIX_ERR_BAD_SIZE;
    *bytes_out = ws_layout(model->cfg, model->hilo_layers, (size_t)max_N, (size_t)max_B).total;
    return RADIX_OK;
}

extern "C" int radix_device_status(void* ws, size_t ws_bytes, void* stream) {
    if (!ws) return RADIX_ERR_NULL_POINTER;
    if (ws_bytes < RADIX_WS_HEADER_BYTES) return RADIX_ERR_WORKSPACE_TOO_SMALL;
    int32_t st = 0;
    HIP_TRY(hipMemcpyAsync(&st, ws, sizeof(st), hipMemcpyDeviceToHost, (hipStream_t)stream));
    HIP_TRY(hipStreamSynchronize((hipStream_t)stream));
    return st;
}

namespace {

int forward_impl(const radix_model* model, const int32_t* tok, const int32_t* pos, const int32_t* cu, int B, int N,
                 int max_seqlen, const int32_t* Is, const int32_t* Ig, int M, bool dedup, bool fused, int pad_to,
                 float* out, void* ws, size_t ws_bytes, hipStream_t stream) {
    const radix_model_config& c = model->cfg;
    fused = fused && dedup && c.compute_dtype != RADIX_F32;   // the fused kernel is the MFMA one
    // the fused kernel addresses the compact q|k|v buffer with 32-bit byte offsets; beyond 4 GB the three-kernel
    // path (same results) takes over
    if (fused && (long long)M * (c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim * (long long)esize(c.compute_dtype) *
                     (model->hilo_layers > 0 ? 2 : 1) >= (1LL << 32))
        fused = false;
    const WsLayout L = ws_layout(c, model->hilo_layers, (size_t)N, (size_t)B);
    if (ws_bytes < L.total) return RADIX_ERR_WORKSPACE_TOO_SMALL;
    char* w = (char*)ws;
    int32_t* hdr = (int32_t*)w;
    hipLaunchKernelGGL(clear_status_kernel, dim3(1), dim3(1), 0, stream, hdr);
    if (N == 0) { HIP_TRY(hipGetLastError()); return RADIX_OK; }
    launch_validate_cu(cu, B, N, max_seqlen, hdr, stream);

    const int dt = c.compute_dtype;          // activation / operand type
    const size_t es = esize(dt);
    const int d = c.d, hd = c.head_dim, dq = c.n_q_heads * hd, dkv = c.n_kv_heads * hd, row = dq + 2 * dkv;
    int32_t* pos_full = (int32_t*)(w + L.pos_full);
    int32_t* ids_c = (int32_t*)(w + L.ids_c);
    int32_t* pos_c = (int32_t*)(w + L.pos_c);
    int32_t* plan = (int32_t*)(w + L.plan);
    float* h = (float*)(w + L.h);
    float* ss = (float*)(w + L.ss);
    void* a = w + L.a;
    void* qkv = w + L.qkv;
    void* qkv_full = dedup ? (void*)(w + L.qkv_full) : qkv;
    void* attn_full = w + L.attn_full;
    void* attn_c = dedup ? (void*)(w + L.attn_c) : attn_full;
    void* mlp = w + L.mlp;
    float* ynorm = (float*)(w + L.ynorm);

    // Performance padding (paper: Implementation Details): the compact space is rounded up to a multiple of
    // pad_to with copies of the first representative, as far as the N rows the workspace holds allow; the
    // padding rows are computed and never scattered.  M_valid = N' keeps indexing the maps.
    const int M_valid = M;
    if (dedup && pad_to > 1) {
        const long long padded = ((long long)M + pad_to - 1) / pad_to * pad_to;
        M = (int)(padded < (long long)N ? padded : (long long)N);
        if (M < M_valid) M = M_valid;
    }

    // Token compaction: positions and ids of the representatives (Algorithm 1, first block)
    if (!pos) {
        launch_default_positions(cu, B, N, pos_full, stream);
        pos = pos_full;
    }
    launch_compact_ids(tok, pos, dedup ? Ig : nullptr, M, M_valid, N, c.vocab, c.max_pos, ids_c, pos_c, hdr, stream);
    launch_embed(model->embed, c.dtype, ids_c, M, d, h, stream);
    if (fused) launch_attn_plan(cu, Is, Ig, B, N, M_valid, c.n_q_heads, c.n_kv_heads, plan, stream);

    // C = A W^T over K columns of A; w_k = row length of W (K, or K / 2 when A rows are (hi, lo) pairs)
    auto gemm = [&](const void* A, const void* W, int Nout, int K, int w_k, int epi, void* o,
                    const QkvEpilogue* qe = nullptr, const ARowMap* amap = nullptr, const NormFusion* nf = nullptr) -> int {
        if (dt != RADIX_F32) return launch_gemm_mfma(A, W, M, Nout, K, epi, o, dt, 0, stream, qe, w_k, amap, nf);
        launch_gemm_f32((const float*)A, (const float*)W, M, Nout, K, epi, (float*)o, stream);
        return RADIX_OK;
    };
    // RMSNorm folded into the GEMMs around it (config.fold_norms; 16-bit operands, d a multiple of 256, layers without
    // (hi, lo) inputs):
    // the projection that last updates the residual rows also writes T(x * gain) and the rows' sums of squares, and
    // the projection that consumes the norm scales its rows by rsqrt(mean + eps).  `normed` says that `a` and `ss`
    // already hold that for the norm about to run.
    const bool can_fold = c.fold_norms == 1 && dt != RADIX_F32 && d % 256 == 0;
    const int n_slots = d / 128;
    bool normed = false;
    NormFusion consume = {};
    consume.ss_in = ss; consume.n_slots_in = n_slots; consume.inv_d = 1.0f / (float)d; consume.eps = c.eps;

    int rc = RADIX_OK;
    for (int l = 0; l < c.n_layers; ++l) {
        const radix_layer_dev& Lw = model->layers[l];
        // leading layers carry every GEMM input (both norm outputs, the attention output, the SwiGLU output) as a
        // 16-bit (hi, lo) pair and multiply over the doubled K against the weights read twice
        const bool hl = l < model->hilo_layers;
        const int w2 = hl ? 2 : 1;
        // timing: the doubled GEMMs of these layers are a category of their own, so that the per-GEMM categories
        // hold launches of one size only
        const int t_qkv = hl ? RADIX_TIME_GEMM_HILO : RADIX_TIME_GEMM_QKV, t_o = hl ? RADIX_TIME_GEMM_HILO : RADIX_TIME_GEMM_O;
        const int t_gu = hl ? RADIX_TIME_GEMM_HILO : RADIX_TIME_GEMM_GATEUP, t_dn = hl ? RADIX_TIME_GEMM_HILO : RADIX_TIME_GEMM_DOWN;
        const bool folded1 = normed;            // the down projection of the layer before prepared this norm
        if (!folded1) {
            TimedScope t(RADIX_TIME_ROWOPS, stream);
            if (hl) {
                if ((rc = launch_rmsnorm_split(h, Lw.g1, M, d, c.eps, a, dt, stream)) != RADIX_OK) return rc;
            } else {
                launch_rmsnorm(h, Lw.g1, M, d, c.eps, a, dt, stream);
            }
        }
        // Q/K-norm and RoPE ride in the QKV GEMM's epilogue when a wavefront block is one head; in a (hi, lo) layer
        // that epilogue also writes q, k and v as (hi, lo) pairs, which attention then multiplies term by term
        const bool fused_rope = dt != RADIX_F32 && hd == 128 && row % 256 == 0;
        const bool qkv_split = hl && fused_rope;
        const int q2 = qkv_split ? 2 : 1;
        {
            TimedScope t(t_qkv, stream);
            const QkvEpilogue qe = {Lw.gq, Lw.gk, model->cos_tab, model->sin_tab, pos_c,
                                    c.n_q_heads, c.n_kv_heads, c.qk_norm, c.eps};
            rc = gemm(a, Lw.wqkv, row, w2 * d, d, qkv_split ? EPI_QKV_ROPE_SPLIT : (fused_rope ? EPI_QKV_ROPE : EPI_STORE), qkv,
                      fused_rope ? &qe : nullptr, nullptr, folded1 ? &consume : nullptr);
            if (rc != RADIX_OK) return rc;
        }
        if (!fused_rope) {
            TimedScope t(RADIX_TIME_ROWOPS, stream);
            launch_qknorm_rope(qkv, dt, M, c.n_q_heads, c.n_kv_heads, hd, c.qk_norm, Lw.gq, Lw.gk, c.eps, pos_c,
                               model->cos_tab, model->sin_tab, stream);
        }
        const size_t attn_row_bytes = (size_t)w2 * dq * es;
        if (fused) {   // scatter, attention and gather in one kernel (exact): compact rows in, compact rows out
            TimedScope t(RADIX_TIME_ATTENTION, stream);
            rc = launch_attention_mfma_fused(qkv, cu, Is, plan, B, N, M_valid, c.n_q_heads, c.n_kv_heads, hd, attn_c,
                                             dt, stream, hl, qkv_split);
            if (rc != RADIX_OK) return rc;
            if (M > M_valid)    // padding rows: any defined value will do, they only feed rows nobody reads
                launch_index_select_rows(attn_c, M_valid, nullptr, M - M_valid, attn_row_bytes,
                                         (char*)attn_c + (size_t)M_valid * attn_row_bytes, hdr, stream, 0);
        }
        if (dedup && !fused) {   // Scatter(q), Scatter(k), Scatter(v): one row copy of the fused q|k|v row
            TimedScope t(RADIX_TIME_SCATTER, stream);
            launch_index_select_rows(qkv, M_valid, Is, N, (size_t)q2 * row * es, qkv_full, hdr, stream);
        }
        if (!fused) {
            TimedScope t(RADIX_TIME_ATTENTION, stream);
            if (dt != RADIX_F32) {
                rc = launch_attention_mfma(qkv_full, cu, B, N, max_seqlen, c.n_q_heads, c.n_kv_heads, hd, attn_full,
                                           dt, stream, hl, qkv_split);
                if (rc != RADIX_OK) return rc;
            } else {
                launch_attention_f32((const float*)qkv_full, cu, B, N, max_seqlen, c.n_q_heads, c.n_kv_heads, hd,
                                     (float*)attn_full, stream);
            }
        }
        // Gather(a): with 16-bit operands the output projection reads its rows through I_gather itself (no copy);
        // the fp32 GEMM, and a full-layout buffer too large for 32-bit row offsets, take the row copy
        const bool gather_in_gemm = dedup && !fused && dt != RADIX_F32 && (long long)N * (long long)attn_row_bytes < (1LL << 32);
        if (dedup && !fused && !gather_in_gemm) {
            TimedScope t(RADIX_TIME_GATHER, stream);
            launch_index_select_rows(attn_full, N, Ig, M, attn_row_bytes, attn_c, hdr, stream, M_valid);
        }
        {
            TimedScope t(t_o, stream);
            const ARowMap amap = {Ig, M_valid, N, hdr};
            const bool fold2 = can_fold && !hl;     // this projection prepares the post-attention norm
            NormFusion produce = {};
            produce.a16 = a; produce.gain = Lw.g2; produce.ss_out = ss;
            rc = gemm(gather_in_gemm ? attn_full : attn_c, Lw.wo, d, w2 * dq, dq, fold2 ? EPI_RESIDUAL_NORM : EPI_RESIDUAL, h,
                      nullptr, gather_in_gemm ? &amap : nullptr, fold2 ? &produce : nullptr);
            if (rc != RADIX_OK) return rc;
            normed = fold2;
        }
        const bool folded2 = normed;
        if (!folded2) {
            TimedScope t(RADIX_TIME_ROWOPS, stream);
            if (hl) {
                if ((rc = launch_rmsnorm_split(h, Lw.g2, M, d, c.eps, a, dt, stream)) != RADIX_OK) return rc;
            } else {
                launch_rmsnorm(h, Lw.g2, M, d, c.eps, a, dt, stream);
            }
        }
        {
            TimedScope t(t_gu, stream);
            rc = gemm(a, Lw.wgu, 2 * c.d_int, w2 * d, d, hl ? EPI_SWIGLU_SPLIT : EPI_SWIGLU, mlp, nullptr, nullptr,
                      folded2 ? &consume : nullptr);
            if (rc != RADIX_OK) return rc;
        }
        {
            TimedScope t(t_dn, stream);
            // prepares the pre-attention norm of the next layer, unless that layer takes (hi, lo) inputs or there is none
            const bool fold1 = can_fold && l + 1 < c.n_layers && l + 1 >= model->hilo_layers;
            NormFusion produce = {};
            produce.a16 = a; produce.ss_out = ss;
            if (fold1) produce.gain = model->layers[l + 1].g1;
            rc = gemm(mlp, Lw.wd, d, w2 * c.d_int, c.d_int, fold1 ? EPI_RESIDUAL_NORM : EPI_RESIDUAL, h, nullptr, nullptr,
                      fold1 ? &produce : nullptr);
            if (rc != RADIX_OK) return rc;
            normed = fold1;
        }
    }
    if (dedup) {
        launch_rmsnorm(h, model->gf, M, d, c.eps, ynorm, RADIX_F32, stream);
        launch_index_select_rows(ynorm, M_valid, Is, N, (size_t)d * 4, out, hdr, stream);   // expand for output
    } else {
        launch_rmsnorm(h, model->gf, M, d, c.eps, out, RADIX_F32, stream);
    }
    HIP_TRY(hipGetLastError());
    return RADIX_OK;
}

int check_common(const radix_model* model, const int32_t* tok, const int32_t* cu, int B, int N, int max_seqlen,
                 const float* out, const void* ws) {
    if (!model || !cu || !ws) return RADIX_ERR_NULL_POINTER;
    if (B < 0 || N < 0 || max_seqlen < 0) return RADIX_ERR_BAD_SIZE;
    if (N > 0 && (!tok || !out)) return RADIX_ERR_NULL_POINTER;
    if (N > 0 && (B == 0 || max_seqlen == 0)) return RADIX_ERR_BAD_SIZE;
    if (B > 65535) return RADIX_ERR_UNSUPPORTED;
    if ((((uintptr_t)ws) & 255) != 0 || (((uintptr_t)out) & 15) != 0) return RADIX_ERR_MISALIGNED;
    return RADIX_OK;
}

}  // namespace

// Whether the deduplicated path runs for a batch (paper: Experiments, radix_mlp_threshold; Limitations,
// "Low-redundancy batches").  Host arithmetic only.
static bool decide_dedup(const radix_model_config& c, int32_t B, int32_t N, int32_t n_compact, const radix_fwd_opts* opts,
                         bool fused) {
    const float threshold = opts ? opts->threshold : RADIX_THRESHOLD_AUTO;
    if (opts && opts->force_dedup != 0) return true;
    if (threshold >= 0.f) return (double)n_compact < (double)threshold * (double)N;
    // automatic: the position-wise work of the N - N' rows saved against what deduplication adds per layer
    const double dq = (double)c.n_q_heads * c.head_dim, dkv = (double)c.n_kv_heads * c.head_dim;
    const double flops_row = 2.0 * c.d * (dq + 2 * dkv) + 2.0 * dq * c.d + 6.0 * (double)c.d * c.d_int;
    const double gemm_rate = c.compute_dtype == RADIX_F32 ? 2.0e13 : 1.1e15;
    const double saved = ((double)N - n_compact) * flops_row / gemm_rate;
    double added;
    if (fused) {
        // the fused kernel starts every workgroup with two more dependent loads (work list, index map) and
        // cuts query blocks where the representatives start, not at multiples of the key tile: about 15 % on
        // top of the attention time when nothing is shared
        const double attn_flops = 2.0 * dq * (double)N * ((double)N / (B > 0 ? B : 1));
        added = 0.15 * attn_flops / 5.0e14;
    } else {
        // three-kernel attention: the scatter of (N' + N) q|k|v rows
        added = ((double)N + n_compact) * (dq + 2 * dkv) * (double)esize(c.compute_dtype) / 5.0e12;
    }
    return n_compact < N && saved > added;
}

static int fused_mode(const radix_model_config& c, const radix_fwd_opts* opts, bool* fused) {
    const int mode = opts ? opts->attention_mode : RADIX_ATTN_AUTO;
    if (mode != RADIX_ATTN_AUTO && mode != RADIX_ATTN_THREE_KERNELS && mode != RADIX_ATTN_FUSED) return RADIX_ERR_BAD_CONFIG;
    if (mode == RADIX_ATTN_FUSED && c.compute_dtype == RADIX_F32) return RADIX_ERR_UNSUPPORTED;
    *fused = mode == RADIX_ATTN_FUSED || (mode == RADIX_ATTN_AUTO && c.compute_dtype != RADIX_F32);
    return RADIX_OK;
}

extern "C" int radix_dedup_decision(const radix_model_config* config, int32_t B, int32_t N, int32_t n_compact,
                                    const radix_fwd_opts* opts, int32_t* dedup_out) {
    if (!config || !dedup_out) return RADIX_ERR_NULL_POINTER;
    if (B < 0 || N < 0 || n_compact < 0 || n_compact > N) return RADIX_ERR_BAD_SIZE;
    const radix_model_config& c = *config;
    int rc = check_config(c);
    if (rc != RADIX_OK) return rc;
    bool fused = false;
    rc = fused_mode(c, opts, &fused);
    if (rc != RADIX_OK) return rc;
    *dedup_out = decide_dedup(c, B, N, n_compact, opts, fused) ? 1 : 0;
    return RADIX_OK;
}

extern "C" int radix_prefill_forward(const radix_model* model, const int32_t* tok, const int32_t* pos,
                                     const int32_t* cu_seqlens, int32_t B, int32_t N, int32_t max_seqlen,
                                     const int32_t* I_scatter, const int32_t* I_gather, int32_t n_compact,
                                     const radix_fwd_opts* opts, float* out, void* ws, size_t ws_bytes, void* stream) {
    int rc = check_common(model, tok, cu_seqlens, B, N, max_seqlen, out, ws);
    if (rc != RADIX_OK) return rc;
    if (n_compact < 0 || n_compact > N || (N > 0 && n_compact == 0)) return RADIX_ERR_BAD_SIZE;
    if (N > 0 && (!I_scatter || !I_gather)) return RADIX_ERR_NULL_POINTER;
    bool fused = false;
    rc = fused_mode(model->cfg, opts, &fused);
    if (rc != RADIX_OK) return rc;
    const bool dedup = decide_dedup(model->cfg, B, N, n_compact, opts, fused);
    if (opts && opts->pad_compact_to < 0) return RADIX_ERR_BAD_CONFIG;
    const int pad_to = opts ? opts->pad_compact_to : 0;
    if (!dedup) n_compact = N;
    return forward_impl(model, tok, pos, cu_seqlens, B, N, max_seqlen, I_scatter, I_gather, n_compact, dedup, fused,
                        pad_to, out, ws, ws_bytes, (hipStream_t)stream);
}

extern "C" int radix_prefill_forward_nodedup(const radix_model* model, const int32_t* tok, const int32_t* pos,
                                             const int32_t* cu_seqlens, int32_t B, int32_t N, int32_t max_seqlen,
                                             float* out, void* ws, size_t ws_bytes, void* stream) {
    int rc = check_common(model, tok, cu_seqlens, B, N, max_seqlen, out, ws);
    if (rc != RADIX_OK) return rc;
    return forward_impl(model, tok, pos, cu_seqlens, B, N, max_seqlen, nullptr, nullptr, N, false, false, 0, out, ws,
                        ws_bytes, (hipStream_t)stream);
}

extern "C" int radix_lm_head_workspace_bytes(const radix_model* model, int32_t max_rows, size_t* bytes_out) {
    if (!model || !bytes_out) return RADIX_ERR_NULL_POINTER;
    if (max_rows < 0) return RADIX_ERR_BAD_SIZE;
    *bytes_out = RADIX_WS_HEADER_BYTES + align_up((size_t)(max_rows ? max_rows : 1) * model->cfg.d * esize(model->cfg.compute_dtype), 256);
    return RADIX_OK;
}

extern "C" int radix_lm_head(const radix_model* model, const float* hidden, int32_t n_src_rows, const int32_t* rows,
                             int32_t n_rows, float* logits, void* ws, size_t ws_bytes, void* stream_) {
    if (!model || !ws) return RADIX_ERR_NULL_POINTER;
    if (n_src_rows < 0 || n_rows < 0) return RADIX_ERR_BAD_SIZE;
    if (!rows && n_rows > n_src_rows) return RADIX_ERR_BAD_SIZE;
    if (!model->lm_head) return RADIX_ERR_UNSUPPORTED;
    const radix_model_config& c = model->cfg;
    size_t need = 0;
    radix_lm_head_workspace_bytes(model, n_rows, &need);
    if (ws_bytes < need) return RADIX_ERR_WORKSPACE_TOO_SMALL;
    if ((((uintptr_t)ws) & 255) != 0 || (((uintptr_t)logits) & 15) != 0) return RADIX_ERR_MISALIGNED;
    hipStream_t stream = (hipStream_t)stream_;
    int32_t* hdr = (int32_t*)ws;
    hipLaunchKernelGGL(clear_status_kernel, dim3(1), dim3(1), 0, stream, hdr);
    if (n_rows == 0) { HIP_TRY(hipGetLastError()); return RADIX_OK; }
    if (!hidden || !logits) return RADIX_ERR_NULL_POINTER;
    if (n_src_rows == 0) return RADIX_ERR_BAD_SIZE;
    void* a = (char*)ws + RADIX_WS_HEADER_BYTES;
    const int dt = c.compute_dtype;
    launch_rows_to_operand(hidden, n_src_rows, rows, n_rows, c.d, a, dt, hdr, stream);
    if (dt == RADIX_F32) {
        launch_gemm_f32((const float*)a, (const float*)model->lm_head, n_rows, c.vocab, c.d, EPI_STORE, logits, stream);
    } else {
        const int rc = launch_gemm_mfma(a, model->lm_head, n_rows, c.vocab, c.d, EPI_STORE_F32, logits, dt, 0, stream);
        if (rc != RADIX_OK) return rc;
    }
    HIP_TRY(hipGetLastError());
    return RADIX_OK;
}

extern "C" int radix_timing_enable(uint32_t category_mask, uint32_t every_nth) {
    g_timer.mask = category_mask & ((1u << RADIX_TIMING_CATEGORIES) - 1u);
    g_timer.stride = every_nth ? every_nth : 1;
    for (int c = 0; c < RADIX_TIMING_CATEGORIES; ++c) g_timer.used[c] = g_timer.seen[c] = 0;
    return RADIX_OK;
}

extern "C" int radix_timing_collect(float* total_ms, int32_t* launches) {
    if (!total_ms || !launches) return RADIX_ERR_NULL_POINTER;
    HIP_TRY(hipDeviceSynchronize());
    for (int c = 0; c < RADIX_TIMING_CATEGORIES; ++c) {
        double sum = 0.0;
        for (size_t i = 0; i < g_timer.used[c]; ++i) {
            float ms = 0.f;
            HIP_TRY(hipEventElapsedTime(&ms, g_timer.pool[c][i].first, g_timer.pool[c][i].second));
            sum += ms;
        }
        total_ms[c] = (float)sum;
        launches[c] = (int32_t)g_timer.used[c];
        g_timer.used[c] = 0;
    }
    return RADIX_OK;
}

extern "C" const char* radix_status_string(int status) {
    switch (status) {
        case RADIX_OK: return "ok";
        case RADIX_ERR_NULL_POINTER: return "null pointer argument";
        case RADIX_ERR_BAD_SIZE: return "bad size argument";
        case RADIX_ERR_UNSUPPORTED: return "unsupported shape, head_dim or dtype";
        case RADIX_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
        case RADIX_ERR_MISALIGNED: return "misaligned pointer";
        case RADIX_ERR_BAD_CU_SEQLENS: return "cu_seqlens is not a non-decreasing array from 0 to N";
        case RADIX_ERR_BAD_TOKEN: return "token id, position id or index out of range";
        case RADIX_ERR_HIP: return "HIP runtime error";
        case RADIX_ERR_BAD_CONFIG: return "inconsistent model configuration";
        case RADIX_ERR_STATIC_LIMIT: return "more sequences than the static scratch array of radix_build_index_static holds";
        default: return "unknown status";
    }
}
