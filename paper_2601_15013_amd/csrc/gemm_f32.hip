// fp32 GEMM C[M, Nout] = A[M, K] * W[Nout, K]^T for the fp32 model configuration (small,
// parity-oriented).  Plain LDS-tiled FMA kernel: 64x64 output tile, 256 threads, 4x4 outputs
// per thread, K consumed in order so every output element is reduced in the same order
// wherever its row sits in the matrix.
#include "common.h"
#include "kernels.h"

namespace {

constexpr int TM = 64, TN = 64, TK = 16;

template <int EPI>
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float* __restrict__ A, const float* __restrict__ W,
                                                       int M, int Nout, int K, float* __restrict__ out) {
    __shared__ float As[TK][TM + 1];
    __shared__ float Ws[TK][TN + 1];
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;        // 16 x 16 threads
    const int m0 = blockIdx.y * TM, n0 = blockIdx.x * TN;
    // thread's rows: ty*4 .. +3 ; columns: {2 tx, 2 tx + 1, 32 + 2 tx, 33 + 2 tx}
    float acc[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += TK) {
        for (int e = tid; e < TM * TK; e += 256) {
            int r = e / TK, k = e % TK;
            int gm = m0 + r, gk = k0 + k;
            As[k][r] = (gm < M && gk < K) ? A[(size_t)gm * K + gk] : 0.f;
            int gn = n0 + r;
            Ws[k][r] = (gn < Nout && gk < K) ? W[(size_t)gn * K + gk] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < TK; ++k) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[k][ty * 4 + i];
            b[0] = Ws[k][2 * tx]; b[1] = Ws[k][2 * tx + 1]; b[2] = Ws[k][32 + 2 * tx]; b[3] = Ws[k][33 + 2 * tx];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int gm = m0 + ty * 4 + i;
        if (gm >= M) continue;
        if (EPI == EPI_SWIGLU) {
            // tile columns 0..31 are gate, 32..63 the matching up columns
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int oc = (n0 >> 1) + 2 * tx + j;
                if (n0 + 32 + 2 * tx + j < Nout) {
                    const float gte = acc[i][j], up = acc[i][j + 2];
                    out[(size_t)gm * (Nout >> 1) + oc] = gte / (1.0f + expf(-gte)) * up;
                }
            }
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int gn = n0 + (j & 1) + 2 * tx + (j >> 1) * 32;
                if (gn >= Nout) continue;
                float* o = out + (size_t)gm * Nout + gn;
                if (EPI == EPI_RESIDUAL) *o = *o + acc[i][j]; else *o = acc[i][j];
            }
        }
    }
}

}  // namespace

void launch_gemm_f32(const float* A, const float* W, int M, int Nout, int K, int epilogue, float* out,
                     hipStream_t stream) {
    if (M <= 0 || Nout <= 0) return;
    dim3 grid(ceil_div(Nout, TN), ceil_div(M, TM)), block(256);
    if (epilogue == EPI_STORE)
        hipLaunchKernelGGL(gemm_f32_kernel<EPI_STORE>, grid, block, 0, stream, A, W, M, Nout, K, out);
    else if (epilogue == EPI_RESIDUAL)
        hipLaunchKernelGGL(gemm_f32_kernel<EPI_RESIDUAL>, grid, block, 0, stream, A, W, M, Nout, K, out);
    else
        hipLaunchKernelGGL(gemm_f32_kernel<EPI_SWIGLU>, grid, block, 0, stream, A, W, M, Nout, K, out);
}
