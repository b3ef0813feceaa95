// fp32 causal varlen GQA attention for the fp32 model configuration (small, parity-oriented).
// One wavefront per (query token, query head): keys are visited 64 at a time with an online
// softmax; lane e accumulates output elements e and e + 64 (head_dim <= 128).
// (Paper: Algorithm 1, "FlashAttn(q, k, v, cu_seqlens, causal=True)" on the full layout.)
#include "common.h"
#include "kernels.h"

namespace {

__global__ __launch_bounds__(64) void attention_f32_kernel(const float* __restrict__ qkv, const int32_t* __restrict__ cu,
                                                           int B, int N, int n_q_heads, int n_kv_heads, int hd,
                                                           float* __restrict__ out) {
    __shared__ float qs[128];
    __shared__ float ps[64];
    const int lane = threadIdx.x;
    const int i = blockIdx.x;          // query token (original layout)
    const int h = blockIdx.y;          // query head
    const int g = h / (n_q_heads / n_kv_heads);
    const int dq = n_q_heads * hd, dkv = n_kv_heads * hd;
    const int row = dq + 2 * dkv;
    int lo = 0, hi = B - 1;
    while (lo < hi) {
        int mid = (lo + hi) >> 1;
        if (cu[mid + 1] > i) hi = mid; else lo = mid + 1;
    }
    int start = cu[lo];
    start = start < 0 ? 0 : (start > i ? i : start);    // a malformed cu_seqlens cannot leave the N rows
    const float scale = 1.0f / sqrtf((float)hd);
    for (int e = lane; e < hd; e += 64) qs[e] = qkv[(size_t)i * row + h * hd + e] * scale;
    __syncthreads();
    float m = -INFINITY, l = 0.f, acc0 = 0.f, acc1 = 0.f;
    for (int j0 = start; j0 <= i; j0 += 64) {
        const int j = j0 + lane;
        float s = -INFINITY;
        if (j <= i) {
            const float* kr = qkv + (size_t)j * row + dq + g * hd;
            float dot = 0.f;
            for (int e = 0; e < hd; ++e) dot = fmaf(qs[e], kr[e], dot);
            s = dot;
        }
        const float m_new = fmaxf(m, wave_max(s));
        const float p = (j <= i) ? expf(s - m_new) : 0.f;
        const float alpha = expf(m - m_new);        // m = -inf on the first chunk: alpha = 0
        l = l * alpha + wave_sum(p);
        acc0 *= alpha; acc1 *= alpha;
        m = m_new;
        __syncthreads();
        ps[lane] = p;
        __syncthreads();
        const int cnt = (i - j0 + 1) < 64 ? (i - j0 + 1) : 64;
        for (int t = 0; t < cnt; ++t) {
            const float* vr = qkv + (size_t)(j0 + t) * row + dq + dkv + g * hd;
            const float pt = ps[t];
            if (lane < hd) acc0 = fmaf(pt, vr[lane], acc0);
            if (lane + 64 < hd) acc1 = fmaf(pt, vr[lane + 64], acc1);
        }
    }
    float* o = out + (size_t)i * dq + h * hd;
    if (lane < hd) o[lane] = acc0 / l;
    if (lane + 64 < hd) o[lane + 64] = acc1 / l;
}

}  // namespace

void launch_attention_f32(const float* qkv, const int32_t* cu, int B, int N, int max_seqlen, int n_q_heads,
                          int n_kv_heads, int hd, float* out, hipStream_t stream) {
    (void)max_seqlen;
    if (N <= 0) return;
    hipLaunchKernelGGL(attention_f32_kernel, dim3(N, n_q_heads), dim3(64), 0, stream, qkv, cu, B, N, n_q_heads,
                       n_kv_heads, hd, out);
}
