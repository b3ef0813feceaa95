// 16-bit MFMA GEMM  C[M, Nout] = A[M, K] * W[Nout, K]^T  (fp32 accumulate) with fused epilogues,
// for bf16 or fp16 operands.
//
// These are the position-wise contractions of the method - Q/K/V and O projections and the
// SwiGLU MLP (paper: Background Eq. 5; Algorithm 1 "QKVProj", "OProj", "MLP") - run on the
// compact row count M = N' (or M = N in the no-dedup baseline).  Both operands are K-contiguous
// ("NT" GEMM), which is exactly the per-lane operand layout of v_mfma_f32_32x32x16_{bf16,f16}:
// lane (r = lane % 32, g = lane / 32) supplies 8 consecutive k of row r for k-group g.
//
// Structure
//   * Workgroup tile BM x BN, k-tile 32, 4 or 8 wavefronts (one or two per SIMD) in a WAVES_M x WAVES_N
//     grid; each wavefront owns (BM/WAVES_M) x (BN/WAVES_N) outputs as 32x32 MFMA accumulators.
//   * The product is formed transposed, C^T = W * A^T (weights are the MFMA "A" operand), so a
//     lane owns one output ROW and 4 consecutive columns per register quad: the fp32 epilogues
//     (residual read-modify-write, plain fp32 store) access 16 bytes per lane straight from that
//     layout, the 16-bit ones transpose through LDS and store whole 256-byte row segments.
//   * Global -> LDS goes through global_load_lds_dwordx4 (no VGPR staging): a wavefront fills
//     1 KB of LDS per instruction, lane L landing at byte 16 L; the XOR swizzle that keeps the
//     fragment reads bank-conflict free is therefore applied to the GLOBAL address each lane
//     fetches.  K-tiles travel in pairs through a ring of five or six LDS stages (the two 64-byte
//     halves of a 128-byte line are requested back to back), one barrier per pair, loads spread
//     one per MFMA slice over the pair; details at the main loop.  The
//     load is issued from inline assembly: issued through the compiler builtin, the compiler's
//     wait-count pass makes every later LDS read wait for ALL loads in flight (it cannot prove
//     that the reads of one stage do not alias the fills of the others), which serialises the
//     pipeline.  The only vector-memory waits are the explicit ones in front of the barriers.
//   * K is consumed in order and there is no split-K, so an output element is reduced in the
//     same order wherever its row sits in the matrix: the deduplicated and the no-dedup pass
//     give bit-identical rows.
//   * Ragged M: rows >= M are fetched from row M-1 and never stored.
//   * Workgroups are numbered so that the 8 XCDs (round-robin dispatch) each work on a compact
//     band of row tiles, sweeping the weight tiles in step with the other XCDs (details at the tile
//     assignment), which keeps an XCD's L2 on few A rows and the shared memory-side cache on few W rows.
#include "common.h"
#include "kernels.h"

namespace {

constexpr int BK = 32;            // k-tile: 64 bytes = 4 chunks of 16 bytes per row

// s_waitcnt with only the vector-memory counter constrained (gfx9 encoding: vmcnt = imm[15:14|3:0],
// expcnt = imm[6:4], lgkmcnt = imm[11:8]).
template <int N> __device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt is 6 bits");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}
// the same, and all LDS reads of this wavefront have returned (lgkmcnt = 0)
template <int N> __device__ __forceinline__ void wait_vmcnt_and_lds() {
    static_assert(N >= 0 && N < 64, "vmcnt is 6 bits");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (0 << 8));
}

// Asynchronous 16-byte-per-lane copy global -> LDS: lane L of the wavefront writes LDS bytes
// [lds_base + 16 L, +16).  lds_base must be wave-uniform.  (s_nop: M0 write -> LDS-DMA hazard.)
// The global address is (uniform 64-bit base) + (per-lane 32-bit byte offset).
__device__ __forceinline__ void dma16(const void* base, uint32_t lane_off, uint32_t lds_base) {
    // the base is wave-uniform by construction; readfirstlane states that where the compiler has parked it in
    // vector registers (it must reach the instruction in a scalar register pair)
    const uint64_t b = (uint64_t)(uintptr_t)base;
    // (the builtin returns a signed int: through uint32_t, or a low half with its top bit set would sign-extend
    // over the high half)
    const uint64_t bs = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(b >> 32)) << 32) |
                        (uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)b);
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 ::"v"(lane_off), "s"(bs), "s"(lds_base) : "memory");
}
__device__ __forceinline__ uint32_t lds_addr(const void* p) {
    return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) char*)p;
}

// LDS slot (in 16-byte units) of chunk c of tile row `row`.  Rows are 4 chunks (64 bytes), so rows
// r, r+4, r+8, r+12 start in the same 64-byte window of the 256-byte bank line; XORing the chunk
// index with bits 2..3 of the row sends the 16 lanes that a ds_read_b128 serves per cycle (16
// consecutive rows of one chunk column) to 16 distinct 16-byte bank groups.
__device__ __forceinline__ int swz(int row) { return (row >> 2) & 3; }
__device__ __forceinline__ int slot(int row, int c) { return row * 4 + (c ^ swz(row)); }

template <int DT, int BM, int BN, int WAVES_M, int WAVES_N, int EPI>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N) void gemm_mfma_kernel(const typename Op<DT>::T* __restrict__ A,
                                                                 const typename Op<DT>::T* __restrict__ W, int M,
                                                                 int Nout, int K, void* __restrict__ out_,
                                                                 int tiles_m, int tiles_n, int w_k,
                                                                 QkvEpilogue qe, ARowMap amap, NormFusion nf, int BAND) {
    typedef typename Op<DT>::T T;
    typedef typename Op<DT>::V8 V8;
    typedef typename Op<DT>::V4 V4;
    constexpr int NW = WAVES_M * WAVES_N;                      // wavefronts: 4 (one per SIMD) or 8 (two per SIMD)
    static_assert(NW == 4 || NW == 8, "4 or 8 wavefronts");
    constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
    constexpr int MB = WTM / 32, NB = WTN / 32;
    constexpr int A_LOADS = BM / (16 * NW), B_LOADS = BN / (16 * NW);   // 1 KB wave-loads per wavefront per k-tile
    constexpr int LOADS = A_LOADS + B_LOADS;
    constexpr int STAGE = (BM + BN) * 4;                       // 16-byte slots per stage
    constexpr bool SWIGLU = EPI == EPI_SWIGLU || EPI == EPI_SWIGLU_SPLIT;
    constexpr bool ROPE = EPI == EPI_QKV_ROPE || EPI == EPI_QKV_ROPE_SPLIT;
    constexpr int PARTS = (EPI == EPI_SWIGLU_SPLIT || EPI == EPI_QKV_ROPE_SPLIT) ? 2 : 1;     // (hi, lo) halves of the output row
    static_assert(!SWIGLU || (NB % 2 == 0), "SwiGLU needs gate/up block pairs in one wavefront");
    static_assert(!ROPE || WTN == 128, "Q/K-norm + RoPE epilogue: one wavefront = one 128-wide head");
    static_assert(EPI != EPI_RESIDUAL_NORM || WTN == 128, "sum-of-squares slots are 128 columns = one wavefront");
    static_assert(LOADS * 2 + A_LOADS * 2 < 64, "vmcnt range");

    constexpr int EPI_PITCH = 272;                             // epilogue row pitch in bytes (256 + 16 pad)
    constexpr int EPI_SLOTS = NW * 64 * EPI_PITCH / 16;        // 64 rows per wavefront
    // ring of k-tile stages: six where they fit the 160 KB of LDS (the smaller tiles), else five
    constexpr int NS = (6 * STAGE * 16 <= 160 * 1024) ? 6 : 5;
    constexpr int LDS_SLOTS = NS * STAGE > EPI_SLOTS ? NS * STAGE : EPI_SLOTS;
    __shared__ uint4 lds_all[LDS_SLOTS];

    // ---- tile assignment (gemm_tile_of: XCD-aware bands of row tiles sweeping the column tiles)
    const GemmTile tile = gemm_tile_of((int)blockIdx.x, tiles_m, tiles_n, BAND);
    const int tm = tile.tm, tn = tile.tn;
    const int m0 = tm * BM, n0 = tn * BN;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    const int r = lane & 31, g = lane >> 5;

    // ---- global-load assignment.  Wave-load j of this wavefront fills tile rows
    // [16 (wave + NW j), +16): lane L -> row + L / 4, LDS chunk L % 4, global chunk (L % 4) ^ swz(row).
    // Addresses are (uniform 64-bit tile base, advanced per k-tile) + (per-lane 32-bit byte offset).
    // With a row map (amap.rows != nullptr) row m of the product is row amap.rows[m] of A: the gather in front
    // of the output projection rides in these offsets instead of being a copy kernel of its own.  Rows at or
    // past amap.n_valid (padding of a bucketed compact space) take source row 0; entries outside
    // [0, amap.n_src) are clamped and reported.
    const int lrow = lane >> 2, lpc = lane & 3;
    const int m_last = M - 1 - m0;                              // last valid row of this tile (ragged M)
    uint32_t a_off[A_LOADS], w_off[B_LOADS];
#pragma unroll
    for (int j = 0; j < A_LOADS; ++j) {
        const int row = 16 * (wave + NW * j) + lrow;
        int src = row < m_last ? row : m_last;
        if (amap.rows != nullptr) {
            const int m = m0 + src;
            src = m < amap.n_valid ? amap.rows[m] : 0;
            if (src < 0 || src >= amap.n_src) {
                set_status(amap.status, RADIX_ERR_BAD_TOKEN);
                src = src < 0 ? 0 : amap.n_src - 1;
            }
        }
        a_off[j] = (uint32_t)(((size_t)src * K + 8 * (lpc ^ swz(row))) * sizeof(T));
    }
#pragma unroll
    for (int j = 0; j < B_LOADS; ++j) {
        const int row = 16 * (wave + NW * j) + lrow;
        w_off[j] = (uint32_t)(((size_t)row * w_k + 8 * (lpc ^ swz(row))) * sizeof(T));
    }
    const char* a_base = (const char*)(A + (amap.rows != nullptr ? (size_t)0 : (size_t)m0 * K));
    const char* w_base = (const char*)(W + (size_t)n0 * w_k);
    const int WKT = w_k / BK;       // k-tiles in a weight row; tiles past it wrap (A = [hi | lo] mode)

    f32x16 acc[NB][MB];
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[j][i][e] = 0.f;

    const int KT = K / BK;

    // EPI_QKV_ROPE: position ids of this lane's rows, fetched before the main loop so that the RoPE
    // table rows can be addressed without a dependent load when the epilogue starts
    int rope_pos[MB];
    if (ROPE) {
#pragma unroll
        for (int i = 0; i < MB; ++i) {
            int gm = m0 + wm * WTM + i * 32 + r;
            gm = gm < M ? gm : M - 1;
            rope_pos[i] = qe.pos_c[gm];
        }
    }

    // RMSNorm folded in (consumer side): the first 16 sum-of-squares slots of every row this lane owns are
    // requested here, ahead of the first tile loads, and added up once those are under way; the row scales
    // then sit in MB registers through the main loop (the epilogue would otherwise start with a chain of
    // dependent loads per tile).
    constexpr bool CONSUMES_NORM = EPI != EPI_RESIDUAL && EPI != EPI_RESIDUAL_NORM && EPI != EPI_STORE_F32;
    constexpr int SS_EARLY = 8;                                 // float2 loads per row requested early
    float2 ssv[MB][SS_EARLY];
    const bool scale_rows = CONSUMES_NORM && nf.ss_in != nullptr;
    if (scale_rows) {
#pragma unroll
        for (int i = 0; i < MB; ++i) {
            int gm = m0 + wm * WTM + i * 32 + r;
            gm = gm < M ? gm : M - 1;
            const float* sp = nf.ss_in + (size_t)gm * nf.n_slots_in;
#pragma unroll
            for (int u = 0; u < SS_EARLY; ++u)
                ssv[i][u] = 2 * u < nf.n_slots_in ? *reinterpret_cast<const float2*>(sp + 2 * u) : make_float2(0.f, 0.f);
        }
    }

    // ---- LDS addressing.  The ring has five stages of STAGE_B bytes; tile t lives in stage t % 5.
    // Stage byte offsets are wave-uniform scalars that rotate as the loop advances, everything
    // lane-dependent is computed once: per k-step ks the byte offset of this lane's chunk in tile row
    // (wave row block) + r; fragment f of the block adds f * 32 rows = f * 2048 bytes.
    constexpr uint32_t STAGE_B = STAGE * 16;
    const char* const lds_c = (const char*)lds_all;
    const uint32_t lds_base = lds_addr(lds_all);
    uint32_t a_rd[2], b_rd[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
        a_rd[ks] = (uint32_t)slot(wm * WTM + r, ks * 2 + g) * 16;
        b_rd[ks] = (uint32_t)(BM * 4 + slot(wn * WTN + r, ks * 2 + g)) * 16;
    }

    // fragment f of a k-step: f < MB is an activation fragment, else a weight fragment
#define RADIX_FRAG1(SO, KS, FA, FB, F)                                                                             \
    do {                                                                                                           \
        if ((F) < MB) {                                                                                            \
            uint4 v = *reinterpret_cast<const uint4*>(lds_c + (SO) + a_rd[KS] + (F) * 2048);                       \
            FA[(F) < MB ? (F) : 0] = *reinterpret_cast<V8*>(&v);                                                   \
        } else {                                                                                                   \
            uint4 v = *reinterpret_cast<const uint4*>(lds_c + (SO) + b_rd[KS] + ((F) - MB) * 2048);                \
            FB[(F) >= MB ? (F) - MB : 0] = *reinterpret_cast<V8*>(&v);                                             \
        }                                                                                                          \
    } while (0)

#define RADIX_DMA1(KT_, SO, F)                                                                                     \
    do {                                                                                                           \
        if ((F) < A_LOADS)                                                                                         \
            dma16(a_base + (size_t)(KT_) * (BK * sizeof(T)), a_off[(F) < A_LOADS ? (F) : 0],                       \
                  lds_base + (SO) + 1024 * (wave + NW * (F)));                                                      \
        else if ((F) < LOADS)                                                                                      \
            dma16(w_base + (size_t)((KT_) >= WKT ? (KT_) - WKT : (KT_)) * (BK * sizeof(T)),                        \
                  w_off[(F) >= A_LOADS && (F) < LOADS ? (F) - A_LOADS : 0],                                        \
                  lds_base + (SO) + BM * 64 + 1024 * (wave + NW * ((F) - A_LOADS)));                                \
    } while (0)

    // loads of k-tiles T0 and T0+1, row group by row group: the two 64-byte halves of every 128-byte
    // line are requested back to back, so the second request merges with the first one's miss in the
    // vector L1 and the line crosses the L2 fabric once (requested a k-tile apart it crosses twice)
#define RADIX_ISSUE2(T0, SA, SB)                                                                                   \
    do {                                                                                                           \
        const int ka__ = (T0) < KT ? (T0) : KT - 2;                                                                \
        _Pragma("unroll") for (int f = 0; f < LOADS; ++f) {                                                        \
            RADIX_DMA1(ka__, SA, f);                                                                               \
            RADIX_DMA1(ka__ + 1, SB, f);                                                                           \
        }                                                                                                          \
    } while (0)

    // MFMAs [lo, hi) of the MB x NB block products of one k-step, in (j, i) order
#define RADIX_MFMA_RANGE(FA, FB, LO, HI)                                                                           \
    do {                                                                                                           \
        _Pragma("unroll") for (int t = (LO); t < (HI); ++t)                                                        \
            acc[t / MB][t % MB] = Op<DT>::mfma(FB[t / MB], FA[t % MB], acc[t / MB][t % MB]);                       \
    } while (0)

    // first k-step of the tile in stage CUR: its MFMAs, led by the fragment reads of its second k-step
#define RADIX_HALF0(CUR)                                                                           \
        _Pragma("unroll") for (int u = 0; u < UNITS; ++u) {                                        \
            RADIX_FRAG1(CUR, 1, fa1, fb1, u);                                                      \
            RADIX_MFMA_RANGE(fa0, fb0, u * HALF / UNITS, (u + 1) * HALF / UNITS);                  \
            __builtin_amdgcn_sched_barrier(0);                                                     \
        }                                                                                          \
        RADIX_MFMA_RANGE(fa0, fb0, HALF, MB * NB);                                                 \
        __builtin_amdgcn_sched_barrier(0);

    constexpr int UNITS = MB + NB;
    constexpr int HALF = MB * NB / 2;      // the reads ride on the first half of a k-step's MFMAs
    static_assert(UNITS >= A_LOADS && UNITS >= B_LOADS, "at most one pair of global->LDS loads per slice");
    // row scales from the sums of squares: slots in increasing order (the early ones, then the rest); adding the
    // zeros that stand in for slots a narrow model does not have changes nothing
    float rsr[MB];
#define RADIX_ROW_SCALES()                                                                                         \
    do {                                                                                                           \
        _Pragma("unroll") for (int i = 0; i < MB; ++i) rsr[i] = 1.0f;                                              \
        if (scale_rows) {                                                                                          \
            _Pragma("unroll") for (int i = 0; i < MB; ++i) {                                                       \
                float ssum = 0.f;                                                                                  \
                _Pragma("unroll") for (int u = 0; u < SS_EARLY; ++u) { ssum += ssv[i][u].x; ssum += ssv[i][u].y; } \
                if (nf.n_slots_in > 2 * SS_EARLY) {                                                                \
                    int gm = m0 + wm * WTM + i * 32 + r;                                                           \
                    gm = gm < M ? gm : M - 1;                                                                      \
                    const float* sp = nf.ss_in + (size_t)gm * nf.n_slots_in;                                       \
                    for (int k0 = 2 * SS_EARLY; k0 < nf.n_slots_in; k0 += 2 * SS_EARLY) {                          \
                        float2 more[SS_EARLY];                                                                     \
                        _Pragma("unroll") for (int u = 0; u < SS_EARLY; ++u)                                       \
                            more[u] = k0 + 2 * u < nf.n_slots_in ? *reinterpret_cast<const float2*>(sp + k0 + 2 * u) \
                                                                 : make_float2(0.f, 0.f);                          \
                        _Pragma("unroll") for (int u = 0; u < SS_EARLY; ++u) { ssum += more[u].x; ssum += more[u].y; } \
                    }                                                                                              \
                }                                                                                                  \
                rsr[i] = 1.0f / sqrtf(ssum * nf.inv_d + nf.eps);                                                   \
            }                                                                                                      \
        }                                                                                                          \
    } while (0)
    V8 fa0[MB], fb0[NB], fa1[MB], fb1[NB];
    if constexpr (NS == 5) {
    RADIX_ISSUE2(0, 0u, STAGE_B);
    {   // activation half of the pair (2, 3); K = 64: tiles 0, 1 again, into stages nobody reads
        const int ka = 2 < KT ? 2 : KT - 2;
#pragma unroll
        for (int f = 0; f < A_LOADS; ++f) {
            RADIX_DMA1(ka, 2 * STAGE_B, f);
            RADIX_DMA1(ka + 1, 3 * STAGE_B, f);
        }
    }
    wait_vmcnt<A_LOADS * 2>();
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int u = 0; u < UNITS; ++u) RADIX_FRAG1(0u, 0, fa0, fb0, u);
    RADIX_ROW_SCALES();

    // One k-tile = two k-steps of 16, software-pipelined over two fragment register sets and
    // scheduled by hand (the scheduling barriers pin the order): the first half of a k-step's MFMAs
    // is cut into UNITS slices, each led by one LDS fragment read for the NEXT k-step; the second half
    // of the MFMAs then covers the LDS latency of those reads, so the matrix pipe always has queued work.
    // K-tiles travel in PAIRS (t even, t+1) and their loads are spread thinly over the MFMA stream (a
    // wavefront that has to wait for room in the memory pipeline cannot issue MFMAs meanwhile):
    //   * first k-step of the even tile: the WEIGHT rows of the pair (t+2, t+3);
    //   * between the two k-steps of the odd tile: wait for this wavefront's loads of the pair
    //     (t+2, t+3), barrier (everybody's share has landed and everybody is done with the pair
    //     (t, t+1)), then, along the second k-step, the ACTIVATION rows of the pair (t+4, t+5) into
    //     the stages of tiles t-1 and t.
    // Pairs past the end re-fetch the last pair into stages nobody reads again: no branch in the body.
    uint32_t so_e = 0, so_o = STAGE_B, so_n = 2 * STAGE_B, so_n1 = 3 * STAGE_B, so_ra = 4 * STAGE_B;   // t, t+1, t+2, t+3, t+4
    for (int kt = 0; kt < KT; kt += 2) {
        const int kw = kt + 2 < KT ? kt + 2 : KT - 2;
#pragma unroll
        for (int u = 0; u < UNITS; ++u) {
#pragma unroll
            for (int dd = 0; dd < 2 * B_LOADS; ++dd)        // load dd: row group dd / 2 of tile t+2 + dd % 2
                if (dd * UNITS / (2 * B_LOADS) == u) {
                    if (dd % 2 == 0) RADIX_DMA1(kw, so_n, A_LOADS + dd / 2);
                    else RADIX_DMA1(kw + 1, so_n1, A_LOADS + dd / 2);
                }
            RADIX_FRAG1(so_e, 1, fa1, fb1, u);
            RADIX_MFMA_RANGE(fa0, fb0, u * HALF / UNITS, (u + 1) * HALF / UNITS);
            __builtin_amdgcn_sched_barrier(0);
        }
        RADIX_MFMA_RANGE(fa0, fb0, HALF, MB * NB);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < UNITS; ++u) {
            RADIX_FRAG1(so_o, 0, fa0, fb0, u);
            RADIX_MFMA_RANGE(fa1, fb1, u * HALF / UNITS, (u + 1) * HALF / UNITS);
            __builtin_amdgcn_sched_barrier(0);
        }
        RADIX_MFMA_RANGE(fa1, fb1, HALF, MB * NB);
        __builtin_amdgcn_sched_barrier(0);

        RADIX_HALF0(so_o)
        wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();
        const int ka = kt + 4 < KT ? kt + 4 : KT - 2;
#pragma unroll
        for (int u = 0; u < UNITS; ++u) {
#pragma unroll
            for (int dd = 0; dd < 2 * A_LOADS; ++dd)
                if (dd * UNITS / (2 * A_LOADS) == u) {
                    if (dd % 2 == 0) RADIX_DMA1(ka, so_ra, dd / 2);
                    else RADIX_DMA1(ka + 1, so_e, dd / 2);       // tile t+5 goes where tile t was
                }
            RADIX_FRAG1(so_n, 0, fa0, fb0, u);
            RADIX_MFMA_RANGE(fa1, fb1, u * HALF / UNITS, (u + 1) * HALF / UNITS);
            __builtin_amdgcn_sched_barrier(0);
        }
        RADIX_MFMA_RANGE(fa1, fb1, HALF, MB * NB);
        __builtin_amdgcn_sched_barrier(0);

        // rotate by two stages: t+2 -> t
        so_e = so_n;
        so_o = so_n + STAGE_B == 5 * STAGE_B ? 0u : so_n + STAGE_B;
        so_n = so_o + STAGE_B == 5 * STAGE_B ? 0u : so_o + STAGE_B;
        so_n1 = so_n + STAGE_B == 5 * STAGE_B ? 0u : so_n + STAGE_B;
        so_ra = so_n1 + STAGE_B == 5 * STAGE_B ? 0u : so_n1 + STAGE_B;
    }
    } else {
    // Six stages = three pair slots: the loads of a pair are issued two pair-iterations before they
    // are waited for (one with five stages), which the short k-tiles of the small workgroup tiles need.
    // Iteration p (tiles t = 2p, t+1): weight rows of pair p+2 along the first k-step of the even tile;
    // between the k-steps of the odd tile wait for pair p+1 (pair p+2 may stay in flight), barrier, then
    // the activation rows of pair p+3 into the stages of pair p.
    RADIX_ISSUE2(0, 0u, STAGE_B);
    RADIX_ISSUE2(2, 2 * STAGE_B, 3 * STAGE_B);
    {
        const int ka = 4 < KT ? 4 : KT - 2;
#pragma unroll
        for (int f = 0; f < A_LOADS; ++f) {
            RADIX_DMA1(ka, 4 * STAGE_B, f);
            RADIX_DMA1(ka + 1, 5 * STAGE_B, f);
        }
    }
    wait_vmcnt<LOADS * 2 + A_LOADS * 2>();
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int u = 0; u < UNITS; ++u) RADIX_FRAG1(0u, 0, fa0, fb0, u);
    RADIX_ROW_SCALES();
    uint32_t so_e = 0, so_n = 2 * STAGE_B, so_w = 4 * STAGE_B;      // stages of t, t+2, t+4 (pairs are adjacent)
    for (int kt = 0; kt < KT; kt += 2) {
        const int kw = kt + 4 < KT ? kt + 4 : KT - 2;
#pragma unroll
        for (int u = 0; u < UNITS; ++u) {
#pragma unroll
            for (int dd = 0; dd < 2 * B_LOADS; ++dd)
                if (dd * UNITS / (2 * B_LOADS) == u) {
                    if (dd % 2 == 0) RADIX_DMA1(kw, so_w, A_LOADS + dd / 2);
                    else RADIX_DMA1(kw + 1, so_w + STAGE_B, A_LOADS + dd / 2);
                }
            RADIX_FRAG1(so_e, 1, fa1, fb1, u);
            RADIX_MFMA_RANGE(fa0, fb0, u * HALF / UNITS, (u + 1) * HALF / UNITS);
            __builtin_amdgcn_sched_barrier(0);
        }
        RADIX_MFMA_RANGE(fa0, fb0, HALF, MB * NB);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < UNITS; ++u) {
            RADIX_FRAG1(so_e + STAGE_B, 0, fa0, fb0, u);
            RADIX_MFMA_RANGE(fa1, fb1, u * HALF / UNITS, (u + 1) * HALF / UNITS);
            __builtin_amdgcn_sched_barrier(0);
        }
        RADIX_MFMA_RANGE(fa1, fb1, HALF, MB * NB);
        __builtin_amdgcn_sched_barrier(0);

        RADIX_HALF0(so_e + STAGE_B)
        // the fragment reads just issued come from a stage that other wavefronts refill right after the
        // barrier (activation rows of pair p+3): they must have returned before this wavefront passes it
        wait_vmcnt_and_lds<LOADS * 2>();
        __builtin_amdgcn_s_barrier();
        const int ka = kt + 6 < KT ? kt + 6 : KT - 2;
#pragma unroll
        for (int u = 0; u < UNITS; ++u) {
#pragma unroll
            for (int dd = 0; dd < 2 * A_LOADS; ++dd)
                if (dd * UNITS / (2 * A_LOADS) == u) {
                    if (dd % 2 == 0) RADIX_DMA1(ka, so_e, dd / 2);
                    else RADIX_DMA1(ka + 1, so_e + STAGE_B, dd / 2);
                }
            RADIX_FRAG1(so_n, 0, fa0, fb0, u);
            RADIX_MFMA_RANGE(fa1, fb1, u * HALF / UNITS, (u + 1) * HALF / UNITS);
            __builtin_amdgcn_sched_barrier(0);
        }
        RADIX_MFMA_RANGE(fa1, fb1, HALF, MB * NB);
        __builtin_amdgcn_sched_barrier(0);

        // rotate by one pair slot
        so_e = so_n;
        so_n = so_w;
        so_w = so_w + 2 * STAGE_B == 6 * STAGE_B ? 0u : so_w + 2 * STAGE_B;
    }
    }
#undef RADIX_ROW_SCALES
#undef RADIX_HALF0
#undef RADIX_ISSUE2
#undef RADIX_MFMA_RANGE
#undef RADIX_DMA1
#undef RADIX_FRAG1
    wait_vmcnt<0>();                  // drain the tail loads ...
    __builtin_amdgcn_s_barrier();     // ... and wait until every wavefront is done with the stages

    // ---- epilogue.  acc[j][i] register e holds output row 32 i + r, column 32 j + 8 (e/4) + 4 g + e%4
    // of this wavefront's block: a lane owns a ROW.  To write full 128-byte lines the block goes
    // through LDS in passes of 64 rows: every lane drops its row pieces into a padded row-major
    // buffer private to its wavefront (row pitch 272 bytes), then the wavefront reads the buffer back
    // 16 bytes per lane, 16 lanes per 256-byte row, and does the global access from that layout.
    constexpr int PITCH = EPI_PITCH;
    char* const ebuf = (char*)lds_all + wave * (64 * PITCH);
    static_assert(MB % 2 == 0 && NB % 2 == 0, "passes of 64 rows / 64 columns");

    // The epilogue derives all its addresses from a lane id the compiler cannot see through, so that
    // none of that arithmetic is hoisted above the main loop, where every vector register counts.
    int lane_opaque = lane;
    asm volatile("" : "+v"(lane_opaque));
    {
    const int lane = lane_opaque;
    const int r = lane & 31, g = lane >> 5;

#define RADIX_ACC(J, I, E) (acc[J][I][E] * rsr[I])

    if (EPI == EPI_RESIDUAL_NORM) {
        // fp32 read-modify-write of the residual stream as below, plus, per row: the updated values times the
        // gain of the norm that follows, in the operand type (what the next projection multiplies), and the
        // sum of their squares over this wavefront's 128 columns (in-lane in (j, q, t) order, then the partner
        // lane that holds the other half of the row's columns).  The loads of a row block are all issued before
        // anything of the block before it is stored: written in that order by hand, because with three
        // unrelated pointers in play the compiler may not move a load above a store on its own, and every
        // (load, add, store) step would then pay the memory latency in turn.
        const int slot = (n0 + wn * WTN) >> 7, n_slots = Nout >> 7;
        const float* grow = nf.gain + n0 + wn * WTN;
        f32x4 gn[NB * 4];
#pragma unroll
        for (int jq = 0; jq < NB * 4; ++jq)
            gn[jq] = *reinterpret_cast<const f32x4*>(grow + (jq >> 2) * 32 + 8 * (jq & 3) + 4 * g);
        f32x4 cur[NB * 4], nxt[NB * 4];
        auto load_block = [&](int i, f32x4* v) {
            const int gm = m0 + wm * WTM + i * 32 + r;
            const float* orow = (const float*)out_ + (size_t)(gm < M ? gm : M - 1) * Nout + n0 + wn * WTN;
#pragma unroll
            for (int jq = 0; jq < NB * 4; ++jq)
                v[jq] = *reinterpret_cast<const f32x4*>(orow + (jq >> 2) * 32 + 8 * (jq & 3) + 4 * g);
        };
        load_block(0, cur);
#pragma unroll
        for (int i = 0; i < MB; ++i) {
            if (i + 1 < MB) load_block(i + 1 < MB ? i + 1 : 0, nxt);
            const int gm = m0 + wm * WTM + i * 32 + r;
            const bool live = gm < M;                              // both lanes of a row agree
            float* orow = (float*)out_ + (size_t)(live ? gm : M - 1) * Nout + n0 + wn * WTN;
            T* arow = (T*)nf.a16 + (size_t)(live ? gm : M - 1) * Nout + n0 + wn * WTN;
            float ss = 0.f;
#pragma unroll
            for (int jq = 0; jq < NB * 4; ++jq) {
                const int c = (jq >> 2) * 32 + 8 * (jq & 3) + 4 * g;
                f32x4 v = cur[jq];
                V4 a;
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    v[t] += acc[jq >> 2][i][(jq & 3) * 4 + t];
                    ss += v[t] * v[t];
                    a[t] = (T)(v[t] * gn[jq][t]);
                }
                if (live) {
                    *reinterpret_cast<f32x4*>(orow + c) = v;
                    *reinterpret_cast<V4*>(arow + c) = a;
                }
            }
            ss += __shfl_xor(ss, 32, 64);
            if (live && g == 0) nf.ss_out[(size_t)gm * n_slots + slot] = ss;
#pragma unroll
            for (int jq = 0; jq < NB * 4; ++jq) cur[jq] = nxt[jq];
        }
    } else if (EPI == EPI_RESIDUAL || EPI == EPI_STORE_F32) {
        // fp32 read-modify-write of the residual stream (or a plain fp32 store) straight from the accumulator layout: per
        // instruction 32 rows x 32 contiguous bytes; all loads of a row block are issued before its
        // stores, and nothing has to be converted, so the LDS detour does not pay here.
#pragma unroll
        for (int i = 0; i < MB; ++i) {
            const int gm = m0 + wm * WTM + i * 32 + r;
            if (gm >= M) continue;
            float* orow = (float*)out_ + (size_t)gm * Nout + n0 + wn * WTN;
#pragma unroll
            for (int j = 0; j < NB; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    f32x4* p = reinterpret_cast<f32x4*>(orow + j * 32 + 8 * q + 4 * g);
                    f32x4 v = {0.f, 0.f, 0.f, 0.f};
                    if (EPI == EPI_RESIDUAL) v = *p;
#pragma unroll
                    for (int t = 0; t < 4; ++t) v[t] += acc[j][i][q * 4 + t];
                    *p = v;
                }
        }
    } else {
        // 16-bit outputs.  EPI_STORE: 128 output columns per wavefront row (256 bytes);
        // EPI_SWIGLU: gate block j / up block j+1 pairs -> 64 output columns per row (128 bytes);
        // EPI_SWIGLU_SPLIT: the same twice, the rounded value into the left half of the output row and what
        // the rounding dropped into the right half (the down projection then runs over the doubled K).
        constexpr int OUT_COLS = SWIGLU ? WTN / 2 : WTN;
        constexpr int CHUNKS = OUT_COLS / 8;                    // 16-byte chunks per output row
        constexpr int ROWS_PER_INST = 64 / CHUNKS;
        const int orow = lane / CHUNKS, ochunk = lane % CHUNKS;
        const int out_w = SWIGLU ? (Nout >> 1) : Nout;          // logical output width; a (hi, lo) row is twice that
        const int ldo = out_w * PARTS;
        const int ncol0 = SWIGLU ? ((n0 + wn * WTN) >> 1) : (n0 + wn * WTN);
        // Q/K-norm + RoPE: which head this wavefront's columns are, and whether it is rotated (q, k) or not (v)
        const int head = (n0 + wn * WTN) >> 7;
        const bool rope_head = ROPE && head < qe.n_q_heads + qe.n_kv_heads;
        const float* rope_gain = (ROPE && head >= qe.n_q_heads) ? qe.gk : qe.gq;
#pragma unroll
        for (int ip = 0; ip < MB; ip += 2) {
#pragma unroll
          for (int part = 0; part < PARTS; ++part) {
#pragma unroll
            for (int il = 0; il < 2; ++il) {
                char* rowp = ebuf + (il * 32 + r) * PITCH;
                if (SWIGLU) {
#pragma unroll
                    for (int j = 0; j < NB; j += 2)
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            V4 v;
#pragma unroll
                            for (int t = 0; t < 4; ++t) {
                                const float gt = RADIX_ACC(j, ip + il, q * 4 + t), up = RADIX_ACC(j + 1, ip + il, q * 4 + t);
                                // silu(g) * u with the hardware reciprocal (1 ulp) instead of an IEEE division
                                const float y = gt * __builtin_amdgcn_rcpf(1.0f + __expf(-gt)) * up;
                                const T hi = (T)y;
                                v[t] = part == 0 ? hi : (T)(y - (float)hi);
                            }
                            *reinterpret_cast<V4*>(rowp + ((j >> 1) * 32 + 8 * q + 4 * g) * 2) = v;
                        }
                } else if (ROPE && rope_head) {
                    // This wavefront's 128 columns are exactly one q or k head of the fused q|k|v row and
                    // a lane owns a row: the per-head RMSNorm is an in-lane sum of 64 squares plus one
                    // exchange with lane ^ 32, and the rotary partner of column c < 64 (block j) is
                    // column c + 64 (block j + 2) of the same lane and register.  (Paper: Q/K norms and
                    // RoPE are position-wise, hence run on compact rows - "Integration with Attention".)
                    const int i = ip + il;
                    float rs = 1.0f;
                    if (qe.qk_norm) {
                        float ss = 0.f;
#pragma unroll
                        for (int j = 0; j < NB; ++j)
#pragma unroll
                            for (int e = 0; e < 16; ++e) ss += RADIX_ACC(j, i, e) * RADIX_ACC(j, i, e);
                        ss += __shfl_xor(ss, 32, 64);
                        rs = 1.0f / sqrtf(ss * (1.0f / 128.0f) + qe.eps);
                    }
                    const float* ct = qe.cos_tab + (size_t)rope_pos[i] * 64;
                    const float* st = qe.sin_tab + (size_t)rope_pos[i] * 64;
#pragma unroll
                    for (int j = 0; j < 2; ++j)
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const int c = 32 * j + 8 * q + 4 * g;
                            const f32x4 cs = *reinterpret_cast<const f32x4*>(ct + c);
                            const f32x4 sn = *reinterpret_cast<const f32x4*>(st + c);
                            f32x4 ga = {1.f, 1.f, 1.f, 1.f}, gb = {1.f, 1.f, 1.f, 1.f};
                            if (qe.qk_norm) {
                                ga = *reinterpret_cast<const f32x4*>(rope_gain + c);
                                gb = *reinterpret_cast<const f32x4*>(rope_gain + c + 64);
                            }
                            V4 va, vb;
#pragma unroll
                            for (int t = 0; t < 4; ++t) {
                                const float xa = RADIX_ACC(j, i, q * 4 + t) * rs * ga[t];
                                const float xb = RADIX_ACC(j + 2, i, q * 4 + t) * rs * gb[t];
                                const float ya = xa * cs[t] - xb * sn[t], yb = xb * cs[t] + xa * sn[t];
                                const T ha = (T)ya, hb = (T)yb;
                                va[t] = part == 0 ? ha : (T)(ya - (float)ha);
                                vb[t] = part == 0 ? hb : (T)(yb - (float)hb);
                            }
                            *reinterpret_cast<V4*>(rowp + c * 2) = va;
                            *reinterpret_cast<V4*>(rowp + (c + 64) * 2) = vb;
                        }
                    __builtin_amdgcn_sched_barrier(0);
                } else {
#pragma unroll
                    for (int j = 0; j < NB; ++j)
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            V4 v;
#pragma unroll
                            for (int t = 0; t < 4; ++t) {
                                const float y = RADIX_ACC(j, ip + il, q * 4 + t);
                                const T hi = (T)y;
                                v[t] = part == 0 ? hi : (T)(y - (float)hi);
                            }
                            *reinterpret_cast<V4*>(rowp + (j * 32 + 8 * q + 4 * g) * 2) = v;
                        }
                }
            }
#pragma unroll
            for (int t = 0; t < 64 / ROWS_PER_INST; ++t) {
                const int row = orow + ROWS_PER_INST * t;
                const int gm = m0 + wm * WTM + ip * 32 + row;
                const uint4 v = *reinterpret_cast<const uint4*>(ebuf + row * PITCH + ochunk * 16);
                if (gm < M)
                    *reinterpret_cast<uint4*>((T*)out_ + (size_t)gm * ldo + part * out_w + ncol0 + ochunk * 8) = v;
            }
          }
        }
    }
#undef RADIX_ACC
    }
}

template <int DT, int BM, int BN, int WAVES_M, int WAVES_N>
int launch_cfg(const void* A, const void* W, int M, int Nout, int K, int w_k, int epilogue, void* out,
               const QkvEpilogue& qe, const ARowMap& amap, const NormFusion& nf, hipStream_t stream) {
    typedef typename Op<DT>::T T;
    if (Nout % BN != 0 || K % (2 * BK) != 0) return RADIX_ERR_UNSUPPORTED;
    const int tiles_m = ceil_div(M, BM), tiles_n = Nout / BN;
    dim3 grid((unsigned)(tiles_m * tiles_n)), block(64 * WAVES_M * WAVES_N);
    const int band_cfg = gemm_band_rows(BM, K, (int)sizeof(T), tiles_n);
#define RADIX_LAUNCH(E)                                                                                       \
    do {                                                                                                      \
        auto kfn = gemm_mfma_kernel<DT, BM, BN, WAVES_M, WAVES_N, E>;                                         \
        hipLaunchKernelGGL(kfn, grid, block, 0, stream, (const T*)A, (const T*)W, M, Nout, K, out, tiles_m,   \
                           tiles_n, w_k, qe, amap, nf, band_cfg);                                             \
    } while (0)
    if (epilogue == EPI_STORE) RADIX_LAUNCH(EPI_STORE);
    else if (epilogue == EPI_RESIDUAL) RADIX_LAUNCH(EPI_RESIDUAL);
    else if (epilogue == EPI_SWIGLU) RADIX_LAUNCH(EPI_SWIGLU);
    else if (epilogue == EPI_SWIGLU_SPLIT) RADIX_LAUNCH(EPI_SWIGLU_SPLIT);
    else if (epilogue == EPI_STORE_F32) RADIX_LAUNCH(EPI_STORE_F32);
    else if (epilogue == EPI_RESIDUAL_NORM) {
        if constexpr (BN / WAVES_N == 128 && WAVES_M * WAVES_N == 4) RADIX_LAUNCH(EPI_RESIDUAL_NORM);
        else return RADIX_ERR_UNSUPPORTED;
    }
    else if (epilogue == EPI_QKV_ROPE) {
        if constexpr (BN / WAVES_N == 128) RADIX_LAUNCH(EPI_QKV_ROPE);
        else return RADIX_ERR_UNSUPPORTED;
    } else if (epilogue == EPI_QKV_ROPE_SPLIT) {
        if constexpr (BN / WAVES_N == 128) RADIX_LAUNCH(EPI_QKV_ROPE_SPLIT);
        else return RADIX_ERR_UNSUPPORTED;
    } else return RADIX_ERR_UNSUPPORTED;
#undef RADIX_LAUNCH
    return RADIX_OK;
}

template <int DT>
int launch_dt(const void* A, const void* W, int M, int Nout, int K, int w_k, int epilogue, void* out, int variant,
              const QkvEpilogue& qe, const ARowMap& amap, const NormFusion& nf, hipStream_t stream) {
    // Tile choice by a small cost model: workgroups run one per CU in rounds, a round costs a fixed part
    // (launch, first loads, epilogue) plus the k-tiles at the rate measured for that shape (microseconds per
    // 32-wide k-tile on MI355X, random fp16 operands): a launch that does not fill its last round pays for it
    // in full, which is what decides between the shapes for small M * Nout.  Eight wavefronts (two per SIMD,
    // 256 registers each) lose nothing in the main loop and overlap each other's epilogue and first loads:
    // 1 to 4 us less per round; the four-wavefront tile is only chosen at K > 16000.
    if (variant == 0) {
        static int n_cu = 0;
        if (n_cu == 0) {
            int dev = 0, cus = 0;
            if (hipGetDevice(&dev) != hipSuccess ||
                hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
                cus = 256;
            n_cu = cus;
        }
        struct Shape { int variant, bm, bn, wave_cols; double fixed_us, ktile_us; };
        static const Shape shapes[5] = {{4, 256, 256, 128, 8.0, 0.832}, {1, 256, 256, 128, 9.0, 0.83},
                                        {5, 128, 256, 64, 6.5, 0.54},   {3, 128, 256, 128, 7.0, 0.57},
                                        {2, 128, 128, 64, 5.0, 0.29}};
        double best = 0.0;
        for (const Shape& sh : shapes) {
            if (Nout % sh.bn != 0) continue;
            if ((epilogue == EPI_QKV_ROPE || epilogue == EPI_QKV_ROPE_SPLIT || epilogue == EPI_RESIDUAL_NORM) &&
                sh.wave_cols != 128)
                continue;                                            // need 128-wide wavefront blocks
            if (epilogue == EPI_RESIDUAL_NORM && sh.variant == 4) continue;   // that epilogue needs 512 registers
            const double tiles = (double)ceil_div(M, sh.bm) * (Nout / sh.bn);
            double rounds = tiles / n_cu;
            if (rounds < 8.0) rounds = (double)(long long)(rounds + 0.999999);   // few rounds: the last one counts whole
            const double t = rounds * (sh.fixed_us + (K / BK) * sh.ktile_us);
            if (variant == 0 || t < best) { best = t; variant = sh.variant; }
        }
        if (variant == 0) return RADIX_ERR_UNSUPPORTED;
    }
    if (variant == 5 && Nout % 256 == 0) return launch_cfg<DT, 128, 256, 2, 4>(A, W, M, Nout, K, w_k, epilogue, out, qe, amap, nf, stream);
    if (variant == 4 && Nout % 256 == 0) return launch_cfg<DT, 256, 256, 4, 2>(A, W, M, Nout, K, w_k, epilogue, out, qe, amap, nf, stream);
    if (variant == 1 && Nout % 256 == 0) return launch_cfg<DT, 256, 256, 2, 2>(A, W, M, Nout, K, w_k, epilogue, out, qe, amap, nf, stream);
    if (variant == 3 && Nout % 256 == 0) return launch_cfg<DT, 128, 256, 2, 2>(A, W, M, Nout, K, w_k, epilogue, out, qe, amap, nf, stream);
    return launch_cfg<DT, 128, 128, 2, 2>(A, W, M, Nout, K, w_k, epilogue, out, qe, amap, nf, stream);
}

}  // namespace

int launch_gemm_mfma(const void* A, const void* W, int M, int Nout, int K, int epilogue, void* out, int op_dtype,
                     int variant, hipStream_t stream, const QkvEpilogue* qkv, int w_k, const ARowMap* a_rows,
                     const NormFusion* norm) {
    if (M <= 0 || Nout <= 0) return RADIX_OK;
    if (K <= 0) return RADIX_ERR_UNSUPPORTED;
    if (w_k == 0) w_k = K;
    if (w_k != K && (2 * w_k != K || w_k % (2 * BK) != 0)) return RADIX_ERR_UNSUPPORTED;
    if ((((uintptr_t)A | (uintptr_t)W | (uintptr_t)out) & 15) != 0) return RADIX_ERR_MISALIGNED;
    QkvEpilogue qe = {};
    if (epilogue == EPI_QKV_ROPE || epilogue == EPI_QKV_ROPE_SPLIT) {
        if (!qkv || Nout % 256 != 0) return RADIX_ERR_UNSUPPORTED;
        qe = *qkv;
    }
    ARowMap amap = {};
    if (a_rows && a_rows->rows) {
        // per-lane 32-bit byte offsets now span the whole source matrix
        if (a_rows->n_src <= 0 || (long long)a_rows->n_src * K * 2 >= (1LL << 32)) return RADIX_ERR_UNSUPPORTED;
        amap = *a_rows;
    }
    NormFusion nf = {};
    if (norm) nf = *norm;
    if (epilogue == EPI_RESIDUAL_NORM) {
        if (Nout % 256 != 0 || !nf.a16 || !nf.gain || !nf.ss_out) return RADIX_ERR_UNSUPPORTED;
        if ((((uintptr_t)nf.a16 | (uintptr_t)nf.gain) & 15) != 0) return RADIX_ERR_MISALIGNED;
    }
    if (nf.ss_in && (nf.n_slots_in <= 0 || nf.n_slots_in % 2 != 0 || ((uintptr_t)nf.ss_in & 7) != 0)) return RADIX_ERR_UNSUPPORTED;
    if (op_dtype == RADIX_BF16) return launch_dt<RADIX_BF16>(A, W, M, Nout, K, w_k, epilogue, out, variant, qe, amap, nf, stream);
    if (op_dtype == RADIX_F16) return launch_dt<RADIX_F16>(A, W, M, Nout, K, w_k, epilogue, out, variant, qe, amap, nf, stream);
    return RADIX_ERR_UNSUPPORTED;
}

// Host-side views of the tile numbering, for tests (declared in radixmlp_bench.h).
extern "C" int radix_debug_gemm_tile(int32_t bid, int32_t tiles_m, int32_t tiles_n, int32_t band, int32_t* tm, int32_t* tn) {
    if (!tm || !tn) return RADIX_ERR_NULL_POINTER;
    if (tiles_m <= 0 || tiles_n <= 0 || band <= 0 || bid < 0 || (long long)bid >= (long long)tiles_m * tiles_n) return RADIX_ERR_BAD_SIZE;
    const GemmTile t = gemm_tile_of(bid, tiles_m, tiles_n, band);
    *tm = t.tm;
    *tn = t.tn;
    return RADIX_OK;
}
extern "C" int radix_debug_gemm_band(int32_t tile_rows, int32_t K, int32_t tiles_n) {
    if (tile_rows <= 0 || K <= 0 || tiles_n <= 0) return RADIX_ERR_BAD_SIZE;
    return gemm_band_rows(tile_rows, K, 2, tiles_n);
}
