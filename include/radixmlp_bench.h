/*
 * radixmlp_bench.h - benchmark instrumentation of libradixmlp, kept apart from the product ABI
 * (radixmlp.h): per-kernel timing with HIP events on the caller's stream.
 */
#ifndef RADIXMLP_BENCH_H
#define RADIXMLP_BENCH_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Optional per-kernel timing for benchmarks.  While a category's bit is set in category_mask,
 * the forward calls bracket every every_nth-th launch of that category (0 or 1: every launch) with a
 * pair of HIP events recorded on the caller's stream; an event pair costs a few microseconds of idle
 * GPU around the launch it brackets, so timing inside a timed region should sample sparsely when
 * launches are short.  radix_timing_collect waits for the device, writes for every category the
 * summed elapsed milliseconds and the number of timed launches since the last collect/enable
 * (arrays of RADIX_TIMING_CATEGORIES entries, HOST pointers) and resets the counters.
 * Process-wide state, not thread-safe; meant for one benchmarking thread.  Mask 0 disables.
 */
enum {
    RADIX_TIME_GEMM_QKV = 0,
    RADIX_TIME_GEMM_O = 1,
    RADIX_TIME_GEMM_GATEUP = 2,
    RADIX_TIME_GEMM_DOWN = 3,
    RADIX_TIME_ATTENTION = 4,
    RADIX_TIME_SCATTER = 5,
    RADIX_TIME_GATHER = 6,
    RADIX_TIME_ROWOPS = 7,
    RADIX_TIME_GEMM_HILO = 8,      /* every GEMM of a layer that runs with (hi, lo) inputs (doubled K) */
    RADIX_TIMING_CATEGORIES = 9
};
int radix_timing_enable(uint32_t category_mask, uint32_t every_nth);
int radix_timing_collect(float* total_ms_host, int32_t* launches_host);

/*
 * Host-side views of the GEMM launch geometry, for tests (no GPU is touched).
 * radix_debug_gemm_tile: the output tile (*tm, *tn) that workgroup `bid` of a launch of tiles_m x tiles_n
 * workgroups computes when row tiles are grouped in bands of `band` - the same function the kernel calls.
 * radix_debug_gemm_band: the band width the launcher picks for 16-bit operands, row tiles of tile_rows rows and
 * rows of K elements (>= 1), or a negative status.
 */
int radix_debug_gemm_tile(int32_t bid, int32_t tiles_m, int32_t tiles_n, int32_t band, int32_t* tm, int32_t* tn);
int radix_debug_gemm_band(int32_t tile_rows, int32_t K, int32_t tiles_n);

#ifdef __cplusplus
}
#endif
#endif /* RADIXMLP_BENCH_H */
