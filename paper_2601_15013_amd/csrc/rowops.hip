// Row-wise, HBM-bound kernels of the compact-space pipeline: gather/scatter (row index-select),
// id/position compaction, embedding lookup, RMSNorm and Q/K-norm + RoPE.
// (Paper: Algorithm 1 "Token Compaction", "Embedding (Compact Space)", "Position Encoding";
//  Implementation Details for the Gather / Scatter operators.)
#include "common.h"
#include "kernels.h"

namespace {

// ------------------------------------------------------------------ index-select of rows
// One wavefront per destination row, 16-byte accesses when the row allows it.  Scatter
// (N' -> N rows) and gather (N -> N' rows) are the same kernel with different index maps.
template <typename V>
__global__ __launch_bounds__(256) void index_select_kernel(const V* __restrict__ src, int n_src_rows,
                                                           const int32_t* __restrict__ idx, int n_rows,
                                                           int n_idx, int row_vecs, V* __restrict__ dst,
                                                           int32_t* status) {
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (row >= n_rows) return;
    int s = row < n_idx ? (idx ? idx[row] : row) : 0;      // padding rows of a bucketed compact space repeat row 0
    if (s < 0 || s >= n_src_rows) {
        if (lane == 0) set_status(status, RADIX_ERR_BAD_TOKEN);
        s = s < 0 ? 0 : n_src_rows - 1;
    }
    const V* sp = src + (size_t)s * row_vecs;
    V* dp = dst + (size_t)row * row_vecs;
    // 8 accesses in flight per lane: all loads of a 512-vector chunk are issued before its stores
    int c = lane;
    for (; c + 7 * 64 < row_vecs; c += 8 * 64) {
        V v[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) v[k] = sp[c + 64 * k];
#pragma unroll
        for (int k = 0; k < 8; ++k) dp[c + 64 * k] = v[k];
    }
    for (; c < row_vecs; c += 64) dp[c] = sp[c];
}

// cu_seqlens must run from 0 to N without decreasing and no sequence may exceed max_seqlen.
__global__ void validate_cu_kernel(const int32_t* __restrict__ cu, int B, int N, int max_seqlen, int32_t* status) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i > B) return;
    const int c = cu[i];
    bool bad = c < 0 || c > N || (i == 0 && c != 0) || (i == B && c != N);
    if (i < B) {
        const int len = cu[i + 1] - c;
        bad = bad || len < 0 || len > max_seqlen;
    }
    if (bad) set_status(status, RADIX_ERR_BAD_CU_SEQLENS);
}

__global__ void default_positions_kernel(const int32_t* __restrict__ cu, int B, int N, int32_t* __restrict__ pos) {
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= N) return;
    int lo = 0, hi = B - 1;
    while (lo < hi) {
        int mid = (lo + hi) >> 1;
        if (cu[mid + 1] > j) hi = mid; else lo = mid + 1;
    }
    pos[j] = j - cu[lo];
}

__global__ void compact_ids_kernel(const int32_t* __restrict__ tok, const int32_t* __restrict__ pos,
                                   const int32_t* __restrict__ Ig, int M, int M_valid, int N, int vocab,
                                   int max_pos, int32_t* __restrict__ ids_c, int32_t* __restrict__ pos_c,
                                   int32_t* status) {
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= M) return;
    // rows past the N' representatives pad the compact space to its bucket: copies of the first representative
    // (paper: Implementation Details, performance padding - "repeat I_gather[0]", and I_gather[0] is token 0)
    int i = j < M_valid ? (Ig ? Ig[j] : j) : 0;
    if (i < 0 || i >= N) { set_status(status, RADIX_ERR_BAD_TOKEN); i = 0; }
    int t = tok[i], p = pos[i];
    if (t < 0 || t >= vocab) { set_status(status, RADIX_ERR_BAD_TOKEN); t = 0; }
    if (p < 0 || p >= max_pos) { set_status(status, RADIX_ERR_BAD_TOKEN); p = 0; }
    ids_c[j] = t;
    pos_c[j] = p;
}

template <typename T>
__global__ __launch_bounds__(256) void embed_kernel(const T* __restrict__ E, const int32_t* __restrict__ ids,
                                                    int M, int d, float* __restrict__ h) {
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (row >= M) return;
    const T* e = E + (size_t)ids[row] * d;
    float* o = h + (size_t)row * d;
    for (int c = lane; c < d; c += 64) o[c] = to_f32<T>(e[c]);
}

// One wavefront per row; the row is read twice (second read hits L2/L1).
template <typename T>
__global__ __launch_bounds__(256) void rmsnorm_kernel(const float* __restrict__ h, const float* __restrict__ g,
                                                      int M, int d, float eps, T* __restrict__ out) {
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (row >= M) return;
    const float* x = h + (size_t)row * d;
    float ss = 0.f;
    for (int c = lane; c < d; c += 64) { float v = x[c]; ss += v * v; }
    ss = wave_sum(ss);
    const float r = 1.0f / sqrtf(ss / (float)d + eps);
    T* o = out + (size_t)row * d;
    for (int c = lane; c < d; c += 64) o[c] = from_f32<T>(x[c] * r * g[c]);
}

// Same, for d = 256 NV: the row stays in registers (NV float4 per lane), so it is read once, with
// 16-byte accesses on both sides.
// SPLIT: the row is written as [hi | lo] (2 d values) with hi = T(y) and lo = T(y - hi), so that a GEMM
// over the doubled K against the weights repeated twice sees the activation to ~2x the significand.
template <typename T, int NV, bool SPLIT>
__global__ __launch_bounds__(256) void rmsnorm_vec_kernel(const float* __restrict__ h, const float* __restrict__ g,
                                                          int M, float eps, T* __restrict__ out) {
    constexpr int d = 256 * NV;
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (row >= M) return;
    const f32x4* x = reinterpret_cast<const f32x4*>(h + (size_t)row * d);
    f32x4 v[NV];
    float ss = 0.f;
#pragma unroll
    for (int k = 0; k < NV; ++k) {
        v[k] = x[lane + 64 * k];
        ss += v[k][0] * v[k][0] + v[k][1] * v[k][1] + v[k][2] * v[k][2] + v[k][3] * v[k][3];
    }
    ss = wave_sum(ss);
    const float r = 1.0f / sqrtf(ss / (float)d + eps);
    const f32x4* gv = reinterpret_cast<const f32x4*>(g);
#pragma unroll
    for (int k = 0; k < NV; ++k) {
        const f32x4 gg = gv[lane + 64 * k];
        T o4[4], l4[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const float y = v[k][t] * r * gg[t];
            o4[t] = from_f32<T>(y);
            l4[t] = from_f32<T>(y - to_f32<T>(o4[t]));
        }
        T* o = out + (size_t)row * (SPLIT ? 2 * d : d) + 4 * (lane + 64 * k);
        if (sizeof(T) == 4) {
            *reinterpret_cast<uint4*>(o) = *reinterpret_cast<uint4*>(o4);
        } else {
            *reinterpret_cast<uint2*>(o) = *reinterpret_cast<uint2*>(o4);
            if (SPLIT) *reinterpret_cast<uint2*>(o + d) = *reinterpret_cast<uint2*>(l4);
        }
    }
}

template <typename T, bool SPLIT>
bool launch_rmsnorm_vec(const float* h, const float* g, int M, int d, float eps, T* out, hipStream_t stream) {
    if (d % 256 != 0 || (((uintptr_t)h | (uintptr_t)g | (uintptr_t)out) & 15) != 0) return false;
    dim3 grid(ceil_div(M, 4)), block(256);
    switch (d / 256) {
#define RADIX_CASE(NV) case NV: hipLaunchKernelGGL((rmsnorm_vec_kernel<T, NV, SPLIT>), grid, block, 0, stream, h, g, M, eps, out); return true;
        RADIX_CASE(1) RADIX_CASE(2) RADIX_CASE(3) RADIX_CASE(4) RADIX_CASE(5) RADIX_CASE(6) RADIX_CASE(8) RADIX_CASE(10)
        RADIX_CASE(12) RADIX_CASE(16) RADIX_CASE(20) RADIX_CASE(32)
#undef RADIX_CASE
        default: return false;
    }
}

// One wavefront per (row, head); lane i < hd/2 owns the rotary pair (i, i + hd/2).
template <typename T>
__global__ __launch_bounds__(256) void qknorm_rope_kernel(T* __restrict__ qkv, int M, int n_q_heads, int n_kv_heads,
                                                          int hd, int qk_norm, const float* __restrict__ gq,
                                                          const float* __restrict__ gk, float eps,
                                                          const int32_t* __restrict__ pos_c,
                                                          const float* __restrict__ cos_tab,
                                                          const float* __restrict__ sin_tab) {
    const int lane = threadIdx.x & 63;
    const int heads = n_q_heads + n_kv_heads;
    const long long item = (long long)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (item >= (long long)M * heads) return;
    const int row = (int)(item / heads), head = (int)(item % heads);
    const int half = hd >> 1;
    const int row_elems = (n_q_heads + 2 * n_kv_heads) * hd;
    T* x = qkv + (size_t)row * row_elems + (size_t)head * hd;   // q heads then k heads are contiguous
    const float* g = head < n_q_heads ? gq : gk;
    const bool act = lane < half;
    float a = act ? to_f32<T>(x[lane]) : 0.f;
    float b = act ? to_f32<T>(x[lane + half]) : 0.f;
    if (qk_norm) {
        float ss = wave_sum(a * a + b * b);
        const float r = 1.0f / sqrtf(ss / (float)hd + eps);
        if (act) { a = a * r * g[lane]; b = b * r * g[lane + half]; }
    }
    if (act) {
        const int p = pos_c[row];
        const float c = cos_tab[(size_t)p * half + lane], s = sin_tab[(size_t)p * half + lane];
        x[lane] = from_f32<T>(a * c - b * s);
        x[lane + half] = from_f32<T>(b * c + a * s);
    }
}

__global__ void bf16_to_f16_kernel(const bf16_t* src, f16_t* dst, size_t n) {   // may run in place
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) dst[i] = (f16_t)(float)src[i];
}

}  // namespace

void launch_bf16_to_f16(const bf16_t* src, f16_t* dst, size_t n, hipStream_t stream) {
    if (n == 0) return;
    const size_t blocks = (n + 255) / 256;
    hipLaunchKernelGGL(bf16_to_f16_kernel, dim3((unsigned)(blocks < 65536 ? blocks : 65536)), dim3(256), 0, stream, src,
                       dst, n);
}

void launch_index_select_rows(const void* src, int n_src_rows, const int32_t* idx, int n_rows, size_t row_bytes,
                              void* dst, int32_t* status, hipStream_t stream, int n_idx) {
    if (n_rows <= 0 || row_bytes == 0) return;
    if (n_idx < 0) n_idx = n_rows;
    const int rows_per_block = 4;
    dim3 grid(ceil_div(n_rows, rows_per_block)), block(256);
    const bool al16 = (row_bytes % 16 == 0) && (((uintptr_t)src | (uintptr_t)dst) % 16 == 0);
    if (al16) {
        hipLaunchKernelGGL(index_select_kernel<uint4>, grid, block, 0, stream, (const uint4*)src, n_src_rows, idx,
                           n_rows, n_idx, (int)(row_bytes / 16), (uint4*)dst, status);
    } else {
        hipLaunchKernelGGL(index_select_kernel<uint32_t>, grid, block, 0, stream, (const uint32_t*)src, n_src_rows,
                           idx, n_rows, n_idx, (int)(row_bytes / 4), (uint32_t*)dst, status);
    }
}

// Row selection + conversion in front of the LM head: one wavefront per output row.
template <typename T>
__global__ void rows_to_operand_kernel(const float* __restrict__ src, int n_src, const int32_t* __restrict__ sel,
                                       int n_rows, int d, T* __restrict__ out, int32_t* __restrict__ status) {
    const int row = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (row >= n_rows) return;
    int s = sel ? sel[row] : row;
    if (s < 0 || s >= n_src) {
        if (lane == 0) set_status(status, RADIX_ERR_BAD_TOKEN);
        s = s < 0 ? 0 : n_src - 1;
    }
    const float* sp = src + (size_t)s * d;
    T* dp = out + (size_t)row * d;
    for (int c = lane; c < d; c += 64) dp[c] = from_f32<T>(sp[c]);
}

void launch_rows_to_operand(const float* src, int n_src, const int32_t* sel, int n_rows, int d, void* out,
                            int out_dtype, int32_t* status, hipStream_t stream) {
    if (n_rows <= 0 || n_src <= 0) return;
    const dim3 grid(ceil_div(n_rows, 4)), block(256);
    if (out_dtype == RADIX_F32)
        hipLaunchKernelGGL(rows_to_operand_kernel<float>, grid, block, 0, stream, src, n_src, sel, n_rows, d, (float*)out, status);
    else if (out_dtype == RADIX_BF16)
        hipLaunchKernelGGL(rows_to_operand_kernel<bf16_t>, grid, block, 0, stream, src, n_src, sel, n_rows, d, (bf16_t*)out, status);
    else
        hipLaunchKernelGGL(rows_to_operand_kernel<f16_t>, grid, block, 0, stream, src, n_src, sel, n_rows, d, (f16_t*)out, status);
}

// ---------------------------------------------------------------- work list of the fused attention kernel
// Per sequence: first representative position (the smallest p with I_gather[I_scatter[start + p]] == start + p,
// or len if the whole sequence duplicates earlier ones; in a trie the predicate is monotone along a sequence - a
// token that opens a new node makes every later token of the sequence open one too - so a binary search finds
// it), the length of the prefix it shares with the sequence before it (compact rows equal, then different: monotone
// as well), and how many 32-row blocks of representative positions go into single-sequence items / are left over.
// Map entries are clamped; a malformed map cannot fault.
__global__ void attn_seq_stats_kernel(const int32_t* __restrict__ cu, const int32_t* __restrict__ Is,
                                      const int32_t* __restrict__ Ig, int B, int N, int M, int slots,
                                      int32_t* __restrict__ first, int32_t* __restrict__ lcp,
                                      int32_t* __restrict__ nfull, int32_t* __restrict__ nrem) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    auto bounds = [&](int s, int& start, int& end) {
        start = cu[s]; end = cu[s + 1];
        start = start < 0 ? 0 : (start > N ? N : start);
        end = end < start ? start : (end > N ? N : end);
    };
    int start, end;
    bounds(b, start, end);
    int lo = 0, hi = end - start;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        int c = Is[start + mid];
        c = c < 0 ? 0 : (c >= M ? M - 1 : c);
        if (Ig[c] == start + mid) hi = mid; else lo = mid + 1;
    }
    first[b] = lo;
    const int blocks = (end - start - lo + 31) / 32;
    nfull[b] = blocks / slots;
    nrem[b] = blocks % slots;
    int common = 0;
    if (b > 0) {
        int ps, pe;
        bounds(b - 1, ps, pe);
        int l2 = 0, h2 = (pe - ps) < (end - start) ? (pe - ps) : (end - start);
        while (l2 < h2) {
            const int mid = (l2 + h2) >> 1;
            if (Is[ps + mid] != Is[start + mid]) h2 = mid; else l2 = mid + 1;
        }
        common = l2;
    }
    lcp[b] = common;
}

// One workgroup: exclusive scans of the two block counts over the sequences, then the item records.
__global__ __launch_bounds__(1024) void attn_plan_kernel(int B, int slots, int max_items, int32_t* __restrict__ plan,
                                                         const int32_t* __restrict__ first,
                                                         const int32_t* __restrict__ lcp, int32_t* nfull,
                                                         int32_t* nrem, int32_t* __restrict__ t_shared,
                                                         int32_t* __restrict__ seq, int32_t* __restrict__ q) {
    __shared__ int wave_tot[2][16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int run_f = 0, run_r = 0;
    for (int base = 0; base < B; base += 1024) {
        const int s = base + tid;
        const int cf = s < B ? nfull[s] : 0, cr = s < B ? nrem[s] : 0;
        int inf = cf, inr = cr;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int vf = __shfl_up(inf, o, 64), vr = __shfl_up(inr, o, 64);
            if (lane >= o) { inf += vf; inr += vr; }
        }
        if (lane == 63) { wave_tot[0][wave] = inf; wave_tot[1][wave] = inr; }
        __syncthreads();
        int bf = 0, br = 0, tf = 0, tr = 0;
#pragma unroll
        for (int w = 0; w < 16; ++w) {
            const int vf = wave_tot[0][w], vr = wave_tot[1][w];
            if (w < wave) { bf += vf; br += vr; }
            tf += vf; tr += vr;
        }
        if (s < B) { nfull[s] = run_f + bf + inf - cf; nrem[s] = run_r + br + inr - cr; }   // now exclusive bases
        run_f += tf; run_r += tr;
        __syncthreads();
    }
    const int n_reg = run_f, n_left = run_r;
    const int n_packed = (n_left + slots - 1) / slots;
    const int n_items = n_reg + n_packed <= max_items ? n_reg + n_packed : max_items;   // cannot exceed it; keeps writes inside
    if (tid == 0) { plan[0] = n_items; plan[1] = n_reg; }
    // records.  Sequence s: its first (leftover) blocks go to the packed items, the rest `slots` at a time.
    for (int s = tid; s < B; s += 1024) {
        const int fb = nfull[s], lb = nrem[s];
        const int cf = (s + 1 < B ? nfull[s + 1] : n_reg) - fb, cr = (s + 1 < B ? nrem[s + 1] : n_left) - lb;
        const int f = first[s];
        for (int i = 0; i < cr; ++i) {
            const int L = lb + i, item = n_reg + L / slots;
            if (item < max_items) { seq[4 * item + L % slots] = s; q[4 * item + L % slots] = f + 32 * i; }
        }
        for (int k = 0; k < cf; ++k) {
            const int item = fb + k;
            if (item >= max_items) break;
            t_shared[item] = 0x7FFFFFFF;
            for (int w = 0; w < 4; ++w) {
                seq[4 * item + w] = w < slots ? s : -1;
                q[4 * item + w] = f + 32 * (cr + k * slots + w);
            }
        }
    }
    for (int L = n_left + tid; L < n_packed * slots; L += 1024) {       // empty slots of the last packed item
        const int item = n_reg + L / slots;
        if (item < max_items) { seq[4 * item + L % slots] = -1; q[4 * item + L % slots] = 0; }
    }
    __syncthreads();
    // packed items: all slots walk together the K/V tiles below the prefix they share (and below every slot's
    // first query, so that the tiles carry no causal boundary of their own)
    for (int g = tid; g < n_packed; g += 1024) {
        const int item = n_reg + g;
        if (item >= max_items) break;
        for (int w = slots; w < 4; ++w) { seq[4 * item + w] = -1; q[4 * item + w] = 0; }
        int common = 0x7FFFFFFF, prev = -1;
        for (int w = 0; w < slots; ++w) {
            const int s = seq[4 * item + w];
            if (s < 0) continue;
            const int qs = q[4 * item + w];
            common = qs < common ? qs : common;
            if (prev >= 0)
                for (int x = prev + 1; x <= s; ++x) common = lcp[x] < common ? lcp[x] : common;
            prev = s;
        }
        t_shared[item] = common == 0x7FFFFFFF ? 0 : common / 64;
    }
}

void launch_attn_plan(const int32_t* cu, const int32_t* Is, const int32_t* Ig, int B, int N, int M, int n_q_heads,
                      int n_kv_heads, int32_t* plan, hipStream_t stream) {
    if (B <= 0 || M <= 0) return;
    const int group = n_q_heads / n_kv_heads;
    const int hpb = (group % 4 == 0) ? 4 : (group % 2 == 0 ? 2 : 1);
    const int slots = 4 / hpb;
    const AttnPlanLayout L = attn_plan_layout((size_t)N, (size_t)B);
    hipLaunchKernelGGL(attn_seq_stats_kernel, dim3(ceil_div(B, 64)), dim3(64), 0, stream, cu, Is, Ig, B, N, M, slots,
                       plan + L.first, plan + L.lcp, plan + L.nfull, plan + L.nrem);
    hipLaunchKernelGGL(attn_plan_kernel, dim3(1), dim3(1024), 0, stream, B, slots, L.max_items, plan, plan + L.first,
                       plan + L.lcp, plan + L.nfull, plan + L.nrem, plan + L.t_shared, plan + L.seq, plan + L.q);
}

void launch_validate_cu(const int32_t* cu, int B, int N, int max_seqlen, int32_t* status, hipStream_t stream) {
    hipLaunchKernelGGL(validate_cu_kernel, dim3(ceil_div(B + 1, 256)), dim3(256), 0, stream, cu, B, N, max_seqlen,
                       status);
}

void launch_default_positions(const int32_t* cu, int B, int N, int32_t* pos_full, hipStream_t stream) {
    if (N <= 0) return;
    hipLaunchKernelGGL(default_positions_kernel, dim3(ceil_div(N, 256)), dim3(256), 0, stream, cu, B, N, pos_full);
}

void launch_compact_ids(const int32_t* tok, const int32_t* pos, const int32_t* Ig, int M, int M_valid, int N,
                        int vocab, int max_pos, int32_t* ids_c, int32_t* pos_c, int32_t* status, hipStream_t stream) {
    if (M <= 0) return;
    hipLaunchKernelGGL(compact_ids_kernel, dim3(ceil_div(M, 256)), dim3(256), 0, stream, tok, pos, Ig, M, M_valid, N,
                       vocab, max_pos, ids_c, pos_c, status);
}

void launch_embed(const void* embed, int dtype, const int32_t* ids_c, int M, int d, float* h, hipStream_t stream) {
    if (M <= 0) return;
    dim3 grid(ceil_div(M, 4)), block(256);
    if (dtype == RADIX_BF16)
        hipLaunchKernelGGL(embed_kernel<bf16_t>, grid, block, 0, stream, (const bf16_t*)embed, ids_c, M, d, h);
    else
        hipLaunchKernelGGL(embed_kernel<float>, grid, block, 0, stream, (const float*)embed, ids_c, M, d, h);
}

int launch_rmsnorm_split(const float* h, const float* g, int M, int d, float eps, void* out, int out_dtype,
                         hipStream_t stream) {
    if (M <= 0) return RADIX_OK;
    if (out_dtype == RADIX_BF16 && launch_rmsnorm_vec<bf16_t, true>(h, g, M, d, eps, (bf16_t*)out, stream)) return RADIX_OK;
    if (out_dtype == RADIX_F16 && launch_rmsnorm_vec<f16_t, true>(h, g, M, d, eps, (f16_t*)out, stream)) return RADIX_OK;
    return RADIX_ERR_UNSUPPORTED;
}

void launch_rmsnorm(const float* h, const float* g, int M, int d, float eps, void* out, int out_dtype,
                    hipStream_t stream) {
    if (M <= 0) return;
    if (out_dtype == RADIX_BF16 && launch_rmsnorm_vec<bf16_t, false>(h, g, M, d, eps, (bf16_t*)out, stream)) return;
    if (out_dtype == RADIX_F16 && launch_rmsnorm_vec<f16_t, false>(h, g, M, d, eps, (f16_t*)out, stream)) return;
    if (out_dtype == RADIX_F32 && launch_rmsnorm_vec<float, false>(h, g, M, d, eps, (float*)out, stream)) return;
    dim3 grid(ceil_div(M, 4)), block(256);
    if (out_dtype == RADIX_BF16)
        hipLaunchKernelGGL(rmsnorm_kernel<bf16_t>, grid, block, 0, stream, h, g, M, d, eps, (bf16_t*)out);
    else if (out_dtype == RADIX_F16)
        hipLaunchKernelGGL(rmsnorm_kernel<f16_t>, grid, block, 0, stream, h, g, M, d, eps, (f16_t*)out);
    else
        hipLaunchKernelGGL(rmsnorm_kernel<float>, grid, block, 0, stream, h, g, M, d, eps, (float*)out);
}

void launch_qknorm_rope(void* qkv, int dtype, int M, int n_q_heads, int n_kv_heads, int hd, int qk_norm,
                        const float* gq, const float* gk, float eps, const int32_t* pos_c, const float* cos_tab,
                        const float* sin_tab, hipStream_t stream) {
    if (M <= 0) return;
    const long long items = (long long)M * (n_q_heads + n_kv_heads);
    dim3 grid((unsigned)((items + 3) / 4)), block(256);
    if (dtype == RADIX_BF16)
        hipLaunchKernelGGL(qknorm_rope_kernel<bf16_t>, grid, block, 0, stream, (bf16_t*)qkv, M, n_q_heads, n_kv_heads,
                           hd, qk_norm, gq, gk, eps, pos_c, cos_tab, sin_tab);
    else if (dtype == RADIX_F16)
        hipLaunchKernelGGL(qknorm_rope_kernel<f16_t>, grid, block, 0, stream, (f16_t*)qkv, M, n_q_heads, n_kv_heads,
                           hd, qk_norm, gq, gk, eps, pos_c, cos_tab, sin_tab);
    else
        hipLaunchKernelGGL(qknorm_rope_kernel<float>, grid, block, 0, stream, (float*)qkv, M, n_q_heads, n_kv_heads,
                           hd, qk_norm, gq, gk, eps, pos_c, cos_tab, sin_tab);
}

extern "C" int radix_index_select_rows(const void* src, int32_t n_src_rows, const int32_t* idx, int32_t n_rows,
                                       size_t row_bytes, void* dst, int32_t* status_dev, void* stream) {
    if (n_rows < 0 || n_src_rows < 0) return RADIX_ERR_BAD_SIZE;
    if (n_rows == 0) return RADIX_OK;
    if (!src || !idx || !dst) return RADIX_ERR_NULL_POINTER;
    if (n_src_rows == 0) return RADIX_ERR_BAD_SIZE;
    if (row_bytes % 4 != 0) return RADIX_ERR_MISALIGNED;
    if ((((uintptr_t)src | (uintptr_t)dst) & 3) != 0) return RADIX_ERR_MISALIGNED;
    launch_index_select_rows(src, n_src_rows, idx, n_rows, row_bytes, dst, status_dev, (hipStream_t)stream);
    HIP_TRY(hipGetLastError());
    return RADIX_OK;
}
