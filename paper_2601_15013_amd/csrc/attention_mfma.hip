// 16-bit (bf16 or fp16 operands) causal varlen GQA attention on the full ragged layout (head_dim = 128), MFMA + online
// softmax.  (Paper: Algorithm 1, "FlashAttn(q, k, v, cu_seqlens, causal=True)"; "Integration
// with Attention": attention is the only step that needs all N rows.)
//
// One workgroup = 4 wavefronts x 32 queries working on ONE KV head: HPB query heads of its GQA
// group (HPB = min(group, 4)) times 128 / HPB query rows, so the K/V tile staged in LDS is shared
// by the query heads of the group and short sequences waste fewer empty query rows.
// Keys/values are walked in tiles of 64 staged in LDS; the next tile's global loads are issued
// before the current tile is multiplied, so their latency overlaps the MFMAs.  Scores are produced TRANSPOSED,
// S^T[key, query] = K * Q^T with v_mfma_f32_32x32x16_{bf16,f16}, so that a lane owns one query column:
// row maxima and sums are in-lane reductions plus one exchange with lane ^ 32, and the running
// rescale factor is a per-lane scalar.  The second product is O^T[hd, query] = V^T * P^T, whose
// B operand is exactly the register layout S^T was produced in (the k index of an MFMA may be
// permuted freely as long as both operands agree), and whose A operand needs V transposed:
// V is transposed once per tile on its way into LDS.
#include "common.h"
#include "kernels.h"

namespace {

constexpr int HD = 128;
constexpr int BKV = 64;     // keys per tile
constexpr int ATT_THREADS = 256;

template <int DT, int HPB>
__global__ __launch_bounds__(ATT_THREADS, 2) void attention_mfma_kernel(const typename Op<DT>::T* __restrict__ qkv,
                                                                     const int32_t* __restrict__ cu, int N,
                                                                     int n_q_heads, int n_kv_heads, int n_qtiles,
                                                                     typename Op<DT>::T* __restrict__ out) {
    typedef typename Op<DT>::T T;
    typedef typename Op<DT>::V8 V8;
    typedef typename Op<DT>::V4 V4;
    __shared__ uint4 Ks[BKV * 16];          // [key][16 chunks of 8 hd], chunk ^= key & 15
    __shared__ uint32_t Vt[HD * 32];        // [hd][32 words of 2 keys], 8-byte chunk ^= (hd >> 1) & 15

    constexpr int BQ = 128 / HPB;                       // query rows per workgroup
    constexpr int WPH = 4 / HPB;                        // wavefronts per query head
    const int seq = blockIdx.z;
    const int qt = n_qtiles - 1 - (int)blockIdx.x;      // heavy (late) tiles first
    // clamped so that a malformed cu_seqlens can never index outside the N rows
    int start = cu[seq], end = cu[seq + 1];
    start = start < 0 ? 0 : (start > N ? N : start);
    end = end < start ? start : (end > N ? N : end);
    const int len = end - start;
    const int q0 = qt * BQ;
    if (q0 >= len) return;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 31, g = lane >> 5;
    const int group = n_q_heads / n_kv_heads;
    const int h = (int)blockIdx.y * HPB + wave / WPH;   // query head of this wavefront
    const int kvh = h / group;                          // same for all wavefronts: HPB divides group
    const int wq = wave % WPH;                          // 32-row slice of the query tile
    const int dq = n_q_heads * HD, dkv = n_kv_heads * HD;
    const size_t row = (size_t)dq + 2 * (size_t)dkv;
    const T* kbase = qkv + (size_t)start * row + dq + (size_t)kvh * HD;
    const T* vbase = kbase + dkv;

    // ---- Q fragment (B operand of S^T = K Q^T): lane (n, g) holds Q[query n][16 ks + 8 g .. +8]
    const int qi = q0 + wq * 32 + n;                    // query offset inside the sequence
    const int qi_c = qi < len ? qi : len - 1;
    V8 qf[8];
    {
        const uint4* qp = (const uint4*)(qkv + (size_t)(start + qi_c) * row + (size_t)h * HD);
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            uint4 v = qp[ks * 2 + g];
            qf[ks] = *reinterpret_cast<V8*>(&v);
        }
    }

    f32x16 o[4];
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int e = 0; e < 16; ++e) o[b][e] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;
    const float sc = 1.4426950408889634f / sqrtf((float)HD);     // log2(e) / sqrt(hd)

    const int wave_qmin = q0 + wq * 32, wave_qmax = wave_qmin + 31;
    const int last_q = (q0 + BQ - 1) < (len - 1) ? (q0 + BQ - 1) : (len - 1);
    const int n_tiles = last_q / BKV + 1;

    // global -> register loads of one K/V tile (rows past the end of the sequence are clamped; the
    // causal mask hides them).  K: thread -> chunk tid % 16 of keys tid / 16 + 16 i.  V: lane -> key
    // pair n, 8 hd columns c8 = wave * 4 + i * 2 + g, so that the transposed store packs 2 keys a word.
    uint4 rk[4], rva[2], rvb[2];
    auto load_tile = [&](int kv0) {
        const int c = tid & 15;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int kr = kv0 + (tid >> 4) + 16 * i;
            kr = kr < len ? kr : len - 1;
            rk[i] = *((const uint4*)(kbase + (size_t)kr * row) + c);
        }
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int c8 = wave * 4 + i * 2 + g;
            int k0r = kv0 + 2 * n, k1r = k0r + 1;
            k0r = k0r < len ? k0r : len - 1;
            k1r = k1r < len ? k1r : len - 1;
            rva[i] = *((const uint4*)(vbase + (size_t)k0r * row) + c8);
            rvb[i] = *((const uint4*)(vbase + (size_t)k1r * row) + c8);
        }
    };
    load_tile(0);

    for (int t = 0; t < n_tiles; ++t) {
        const int kv0 = t * BKV;
        __syncthreads();
        // ---- K tile -> LDS (row-major, swizzled); V tile -> LDS transposed
        {
            const int c = tid & 15;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int key = (tid >> 4) + 16 * i;
                Ks[key * 16 + (c ^ (key & 15))] = rk[i];
            }
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int c8 = wave * 4 + i * 2 + g;
                const uint32_t aw[4] = {rva[i].x, rva[i].y, rva[i].z, rva[i].w};
                const uint32_t bw[4] = {rvb[i].x, rvb[i].y, rvb[i].z, rvb[i].w};
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const uint32_t lo = (aw[e >> 1] >> ((e & 1) * 16)) & 0xFFFFu;
                    const uint32_t hi = (bw[e >> 1] >> ((e & 1) * 16)) & 0xFFFFu;
                    const int hd = c8 * 8 + e;
                    Vt[hd * 32 + (((n >> 1) ^ ((hd >> 1) & 15)) << 1) + (n & 1)] = lo | (hi << 16);
                }
            }
        }
        __syncthreads();
        if (t + 1 < n_tiles) load_tile(kv0 + BKV);     // in flight while this tile is multiplied
        if (kv0 > wave_qmax) continue;          // whole tile is in this wavefront's future

        // ---- S^T = K Q^T : two 32-key blocks
        f32x16 s[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
            for (int e = 0; e < 16; ++e) s[kb][e] = 0.f;
            const int key = kb * 32 + n;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                uint4 v = Ks[key * 16 + ((ks * 2 + g) ^ (key & 15))];
                s[kb] = Op<DT>::mfma(*reinterpret_cast<V8*>(&v), qf[ks], s[kb]);
            }
        }
        // ---- scale, causal mask (register e of block kb is key kv0 + 32 kb + 8 (e/4) + 4 g + e%4)
        const bool need_mask = (kv0 + BKV - 1) > wave_qmin;
        float tmax = -INFINITY;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                float v = s[kb][e] * sc;
                if (need_mask) {
                    const int kj = kv0 + kb * 32 + 8 * (e >> 2) + 4 * g + (e & 3);
                    if (kj > qi_c) v = -INFINITY;
                }
                s[kb][e] = v;
                tmax = fmaxf(tmax, v);
            }
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
        const float m_new = fmaxf(m_run, tmax);       // finite: tile 0 always holds key 0 <= query
        const float alpha = exp2f(m_run - m_new);
        m_run = m_new;
        float psum = 0.f;
        V8 pf[4];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const float p = exp2f(s[kb][e] - m_new);
                psum += p;
                pf[kb * 2 + (e >> 3)][e & 7] = (T)p;
            }
        l_run = l_run * alpha + psum;
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int e = 0; e < 16; ++e) o[b][e] *= alpha;

        // ---- O^T += V^T P^T : 4 hd blocks x 4 k-steps of 16 keys
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const int hd = b * 32 + n;
                const uint2 lo = *reinterpret_cast<const uint2*>(&Vt[hd * 32 + (((4 * kk + g) ^ ((hd >> 1) & 15)) << 1)]);
                const uint2 hi = *reinterpret_cast<const uint2*>(&Vt[hd * 32 + (((4 * kk + 2 + g) ^ ((hd >> 1) & 15)) << 1)]);
                uint4 v = make_uint4(lo.x, lo.y, hi.x, hi.y);
                o[b] = Op<DT>::mfma(*reinterpret_cast<V8*>(&v), pf[kk], o[b]);
            }
        }
    }

    // ---- normalise and store: register e of block b is hd = 32 b + 8 (e/4) + 4 g + e%4
    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    if (qi < len) {
        const float inv = 1.0f / l_tot;
        T* op = out + (size_t)(start + qi) * dq + (size_t)h * HD;
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                V4 v;
#pragma unroll
                for (int j = 0; j < 4; ++j) v[j] = (T)(o[b][q4 * 4 + j] * inv);
                *reinterpret_cast<V4*>(op + b * 32 + q4 * 8 + g * 4) = v;
            }
    }
}

}  // namespace

int launch_attention_mfma(const void* qkv, const int32_t* cu, int B, int N, int max_seqlen, int n_q_heads,
                          int n_kv_heads, int hd, void* out, int op_dtype, hipStream_t stream) {
    if (N <= 0 || B <= 0) return RADIX_OK;
    if (hd != HD) return RADIX_ERR_UNSUPPORTED;
    if (max_seqlen <= 0) return RADIX_ERR_BAD_SIZE;
    if (B > 65535 || n_q_heads > 65535) return RADIX_ERR_UNSUPPORTED;
    if (op_dtype != RADIX_BF16 && op_dtype != RADIX_F16) return RADIX_ERR_UNSUPPORTED;
    const int group = n_q_heads / n_kv_heads;
    const int hpb = (group % 4 == 0) ? 4 : (group % 2 == 0 ? 2 : 1);    // query heads per workgroup
    const int n_qtiles = ceil_div(max_seqlen, 128 / hpb);
    const dim3 grid(n_qtiles, n_q_heads / hpb, B), block(ATT_THREADS);
#define RADIX_ATT(DT, HPB)                                                                                       \
    hipLaunchKernelGGL((attention_mfma_kernel<DT, HPB>), grid, block, 0, stream, (const Op<DT>::T*)qkv, cu, N,   \
                       n_q_heads, n_kv_heads, n_qtiles, (Op<DT>::T*)out)
    if (op_dtype == RADIX_BF16) {
        if (hpb == 4) RADIX_ATT(RADIX_BF16, 4); else if (hpb == 2) RADIX_ATT(RADIX_BF16, 2); else RADIX_ATT(RADIX_BF16, 1);
    } else {
        if (hpb == 4) RADIX_ATT(RADIX_F16, 4); else if (hpb == 2) RADIX_ATT(RADIX_F16, 2); else RADIX_ATT(RADIX_F16, 1);
    }
#undef RADIX_ATT
    return RADIX_OK;
}
