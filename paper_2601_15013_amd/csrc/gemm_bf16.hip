// bf16 MFMA GEMM  C[M, Nout] = A[M, K] * W[Nout, K]^T  (fp32 accumulate) with fused epilogues.
//
// These are the position-wise contractions of the method - Q/K/V and O projections and the
// SwiGLU MLP (paper: Background Eq. 5; Algorithm 1 "QKVProj", "OProj", "MLP") - run on the
// compact row count M = N' (or M = N in the no-dedup baseline).  Both operands are K-contiguous
// ("NT" GEMM), which is exactly the per-lane operand layout of v_mfma_f32_32x32x16_bf16:
// lane (r = lane % 32, g = lane / 32) supplies 8 consecutive k of row r for k-group g.
//
// Structure: workgroup tile BM x BN x 64, 256 threads = 4 wavefronts in a WAVES_M x WAVES_N
// grid, each wavefront owning a (BM/WAVES_M) x (BN/WAVES_N) block of 32x32 MFMA accumulators.
// Global -> registers -> LDS with two LDS stages (one barrier per k-tile); the next k-tile's
// global loads are in flight while the current one is multiplied.  LDS rows are 128 bytes with
// the 16-byte chunk index XOR-swizzled by (row & 7) so that fragment reads and tile writes are
// bank-conflict free.  K is consumed in order and there is no split-K, so an output element is
// reduced in the same order wherever its row sits in the matrix: the deduplicated and the
// no-dedup pass give bit-identical rows.
//
// Ragged M: rows >= M are loaded from row M-1 and never stored.
#include "common.h"
#include "kernels.h"

namespace {

constexpr int BK = 64;            // k-tile (bf16 elements) = 128 bytes = 8 chunks of 16 bytes
constexpr int GEMM_THREADS = 256;

__device__ __forceinline__ int swz(int row, int chunk) { return row * 8 + (chunk ^ (row & 7)); }

template <int BM, int BN, int WAVES_M, int WAVES_N, int EPI>
__global__ __launch_bounds__(GEMM_THREADS) void gemm_bf16_kernel(const bf16_t* __restrict__ A,
                                                                 const bf16_t* __restrict__ W, int M, int Nout, int K,
                                                                 void* __restrict__ out_) {
    static_assert(WAVES_M * WAVES_N == 4, "4 wavefronts");
    constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
    constexpr int MB = WTM / 32, NB = WTN / 32;
    constexpr int A_CH = BM * 8 / GEMM_THREADS, B_CH = BN * 8 / GEMM_THREADS;   // 16-byte chunks per thread
    static_assert(EPI != EPI_SWIGLU || (NB % 2 == 0), "SwiGLU needs gate/up block pairs in one wavefront");

    extern __shared__ uint4 lds[];                  // [2 stages][(BM + BN) * 8 chunks]
    constexpr int STAGE = (BM + BN) * 8;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    const int r = lane & 31, g = lane >> 5;

    // global-load assignment: chunk column tid % 8, rows tid / 8 + 32 i
    const int lc = tid & 7, lr = tid >> 3;
    const uint4* Ag[A_CH];
    const uint4* Wg[B_CH];
#pragma unroll
    for (int i = 0; i < A_CH; ++i) {
        int gm = m0 + lr + 32 * i;
        gm = gm < M ? gm : M - 1;
        Ag[i] = (const uint4*)(A + (size_t)gm * K) + lc;
    }
#pragma unroll
    for (int i = 0; i < B_CH; ++i) Wg[i] = (const uint4*)(W + (size_t)(n0 + lr + 32 * i) * K) + lc;

    f32x16 acc[MB][NB];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    uint4 ra[A_CH], rb[B_CH];
    const int KT = K / BK;
#pragma unroll
    for (int i = 0; i < A_CH; ++i) ra[i] = Ag[i][0];
#pragma unroll
    for (int i = 0; i < B_CH; ++i) rb[i] = Wg[i][0];
#pragma unroll
    for (int i = 0; i < A_CH; ++i) lds[swz(lr + 32 * i, lc)] = ra[i];
#pragma unroll
    for (int i = 0; i < B_CH; ++i) lds[BM * 8 + swz(lr + 32 * i, lc)] = rb[i];
    __syncthreads();

    for (int kt = 0; kt < KT; ++kt) {
        const uint4* sA = lds + (kt & 1) * STAGE;
        const uint4* sB = sA + BM * 8;
        if (kt + 1 < KT) {
#pragma unroll
            for (int i = 0; i < A_CH; ++i) ra[i] = Ag[i][(kt + 1) * 8];
#pragma unroll
            for (int i = 0; i < B_CH; ++i) rb[i] = Wg[i][(kt + 1) * 8];
        }
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8 fa[MB], fb[NB];
            const int ch = ks * 2 + g;
#pragma unroll
            for (int i = 0; i < MB; ++i) {
                uint4 v = sA[swz(wm * WTM + i * 32 + r, ch)];
                fa[i] = *reinterpret_cast<bf16x8*>(&v);
            }
#pragma unroll
            for (int j = 0; j < NB; ++j) {
                uint4 v = sB[swz(wn * WTN + j * 32 + r, ch)];
                fb[j] = *reinterpret_cast<bf16x8*>(&v);
            }
#pragma unroll
            for (int i = 0; i < MB; ++i)
#pragma unroll
                for (int j = 0; j < NB; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < KT) {
            uint4* dA = lds + ((kt + 1) & 1) * STAGE;
            uint4* dB = dA + BM * 8;
#pragma unroll
            for (int i = 0; i < A_CH; ++i) dA[swz(lr + 32 * i, lc)] = ra[i];
#pragma unroll
            for (int i = 0; i < B_CH; ++i) dB[swz(lr + 32 * i, lc)] = rb[i];
        }
        __syncthreads();
    }

    // ---- epilogue.  Accumulator (i, j), register e: row = 8 (e / 4) + 4 g + e % 4, column = r.
#pragma unroll
    for (int i = 0; i < MB; ++i) {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int gm = m0 + wm * WTM + i * 32 + 8 * (e >> 2) + 4 * g + (e & 3);
            if (gm >= M) continue;
            if (EPI == EPI_SWIGLU) {
                bf16_t* out = (bf16_t*)out_;
#pragma unroll
                for (int j = 0; j < NB; j += 2) {
                    const int gn = n0 + wn * WTN + j * 32;              // gate block; up block follows
                    const float gt = acc[i][j][e], up = acc[i][j + 1][e];
                    out[(size_t)gm * (Nout >> 1) + (gn >> 1) + r] = (bf16_t)(gt / (1.0f + __expf(-gt)) * up);
                }
            } else {
#pragma unroll
                for (int j = 0; j < NB; ++j) {
                    const int gn = n0 + wn * WTN + j * 32 + r;
                    if (EPI == EPI_RESIDUAL) {
                        float* o = (float*)out_ + (size_t)gm * Nout + gn;
                        *o = *o + acc[i][j][e];
                    } else {
                        ((bf16_t*)out_)[(size_t)gm * Nout + gn] = (bf16_t)acc[i][j][e];
                    }
                }
            }
        }
    }
}

template <int BM, int BN, int WAVES_M, int WAVES_N>
int launch_cfg(const bf16_t* A, const bf16_t* W, int M, int Nout, int K, int epilogue, void* out, hipStream_t stream) {
    if (Nout % BN != 0 || K % BK != 0) return RADIX_ERR_UNSUPPORTED;
    dim3 grid(Nout / BN, ceil_div(M, BM)), block(GEMM_THREADS);
    const size_t smem = (size_t)2 * (BM + BN) * 8 * sizeof(uint4);
#define RADIX_LAUNCH(E)                                                                                       \
    do {                                                                                                      \
        auto kfn = gemm_bf16_kernel<BM, BN, WAVES_M, WAVES_N, E>;                                             \
        if (smem > 64 * 1024) {                                                                               \
            if (hipFuncSetAttribute((const void*)kfn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem)  \
                != hipSuccess) return RADIX_ERR_HIP;                                                          \
        }                                                                                                     \
        hipLaunchKernelGGL(kfn, grid, block, smem, stream, A, W, M, Nout, K, out);                            \
    } while (0)
    if (epilogue == EPI_STORE) RADIX_LAUNCH(EPI_STORE);
    else if (epilogue == EPI_RESIDUAL) RADIX_LAUNCH(EPI_RESIDUAL);
    else RADIX_LAUNCH(EPI_SWIGLU);
#undef RADIX_LAUNCH
    return RADIX_OK;
}

}  // namespace

int launch_gemm_bf16(const bf16_t* A, const bf16_t* W, int M, int Nout, int K, int epilogue, void* out,
                     hipStream_t stream) {
    if (M <= 0 || Nout <= 0) return RADIX_OK;
    if (K <= 0) return RADIX_ERR_UNSUPPORTED;
    if ((((uintptr_t)A | (uintptr_t)W) & 15) != 0) return RADIX_ERR_MISALIGNED;
    return launch_cfg<128, 128, 2, 2>(A, W, M, Nout, K, epilogue, out, stream);
}
