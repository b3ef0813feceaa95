// Stand-alone timing probe of the MFMA GEMM kernel (not part of the library).  Built by build.py into
// _build/gemm_probe[_no_loads|_no_frags|_no_mfma|_mfma_only] from this file + gemm_mfma.hip; the
// suffixed builds leave out parts of the main loop (see the RADIX_GEMM_PROBE_* switches there), so their
// times show what the loads, the LDS reads and the matrix pipe cost on their own.
//
//   gemm_probe M Nout K epilogue(0 store,1 residual,2 swiglu) data(random|zero) [iters]
//
// data = zero fills both operands with zeros: the MFMA rate depends on the operand bits (switching
// power), which this makes visible.
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include "kernels.h"

#define CK(x)                                                                            \
    do {                                                                                 \
        hipError_t e_ = (x);                                                             \
        if (e_ != hipSuccess) {                                                          \
            printf("hip error %s at line %d\n", hipGetErrorString(e_), __LINE__);        \
            return 1;                                                                    \
        }                                                                                \
    } while (0)

__global__ void probe_fill_kernel(uint16_t* p, size_t n, uint32_t seed, int zero) {
    const size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
    if (i >= n) return;
    uint32_t x = (uint32_t)i * 2654435761u ^ seed;
    x ^= x >> 15; x *= 2246822519u; x ^= x >> 13; x *= 3266489917u; x ^= x >> 16;
    // fp16 bit patterns of moderate magnitude: random sign and mantissa, exponent in [2^-4, 2^-1]
    const uint16_t h = (uint16_t)(((x >> 3) & 0x8000u) | ((11u + (x & 3u)) << 10) | ((x >> 8) & 0x3FFu));
    p[i] = zero ? (uint16_t)0 : h;
}

int main(int argc, char** argv) {
    if (argc < 6) {
        printf("usage: %s M Nout K epilogue(0|1|2) data(random|zero) [iters]\n", argv[0]);
        return 2;
    }
    const int M = atoi(argv[1]), N = atoi(argv[2]), K = atoi(argv[3]), epi = atoi(argv[4]);
    const int zero = strcmp(argv[5], "zero") == 0;
    const int iters = argc > 6 ? atoi(argv[6]) : 20;
    if (M <= 0 || N <= 0 || K <= 0 || epi < 0 || epi > 2 || iters <= 0) return 2;
    const size_t na = (size_t)M * K, nw = (size_t)N * K;
    const size_t out_bytes = (size_t)M * N * 4;      // large enough for every epilogue
    uint16_t *A, *W;
    void* out;
    CK(hipMalloc(&A, na * 2));
    CK(hipMalloc(&W, nw * 2));
    CK(hipMalloc(&out, out_bytes));
    CK(hipMemset(out, 0, out_bytes));
    probe_fill_kernel<<<(unsigned)((na + 255) / 256), 256>>>(A, na, 123u, zero);
    probe_fill_kernel<<<(unsigned)((nw + 255) / 256), 256>>>(W, nw, 77u, zero);
    CK(hipDeviceSynchronize());
    for (int i = 0; i < 3; ++i) {
        const int rc = launch_gemm_mfma(A, W, M, N, K, epi, out, RADIX_F16, 0, 0);
        if (rc) { printf("launch_gemm_mfma: status %d\n", rc); return 1; }
    }
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    CK(hipEventRecord(e0));
    for (int i = 0; i < iters; ++i) launch_gemm_mfma(A, W, M, N, K, epi, out, RADIX_F16, 0, 0);
    CK(hipEventRecord(e1));
    CK(hipEventSynchronize(e1));
    float ms = 0.f;
    CK(hipEventElapsedTime(&ms, e0, e1));
    ms /= iters;
    printf("M=%d Nout=%d K=%d epilogue=%d data=%s  %.1f us  %.1f TFLOP/s\n", M, N, K, epi, zero ? "zero" : "random",
           ms * 1e3, 2.0 * M * N * K / ms / 1e9);
    CK(hipFree(A)); CK(hipFree(W)); CK(hipFree(out));
    return 0;
}
