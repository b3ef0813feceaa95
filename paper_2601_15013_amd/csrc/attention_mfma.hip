// 16-bit (bf16 or fp16 operands) causal varlen GQA attention on the full ragged layout (head_dim = 128),
// MFMA + online softmax.  (Paper: Algorithm 1, "FlashAttn(q, k, v, cu_seqlens, causal=True)";
// "Integration with Attention": attention is the only step that needs all N rows.)
//
// One workgroup = 4 wavefronts x 32 queries working on ONE KV head: HPB query heads of its GQA
// group (HPB = min(group, 4)) times 128 / HPB query rows, so the K/V tile staged in LDS is shared
// by the query heads of the group and short sequences waste fewer empty query rows.
//
// Data path.  K and V tiles of 64 keys go global -> LDS with global_load_lds_dwordx4 (no VGPR
// staging), both row-major [key][128], two stages: the loads of tile t+1 are issued right after the
// barrier that retires tile t-1 and land while tile t is multiplied; one barrier per tile.  The DMA
// writes LDS linearly, so the XOR swizzles that keep the fragment reads bank-conflict free are
// applied to the global address a lane fetches.
//
// Scores are produced TRANSPOSED, S^T[key, query] = K * Q^T with v_mfma_f32_32x32x16_{bf16,f16}, so
// that a lane owns one query column: row maxima and sums are in-lane reductions plus one exchange
// with lane ^ 32, and the running rescale factor is a per-lane scalar.  The second product is
// O^T[hd, query] = V^T * P^T.  Its B operand is exactly the register layout S^T was produced in (the
// k index of an MFMA may be permuted freely as long as both operands agree).  Its A operand needs,
// per lane, 8 keys of one hd column out of the row-major V tile: that is what ds_read_b64_tr_b16
// delivers - 16 lanes hand in the addresses of a 4-key x 16-column block (lane 4 e + a: key e, columns
// 4 a .. 4 a + 3) and lane l receives column l of keys 0..3 - so V is never transposed in memory.
//
// FUSED mode (scatter and gather folded into this kernel; exact).  Q, K and V stay in the COMPACT
// buffer: the row of sequence position p is I_scatter[start + p], looked up one tile ahead of the
// K/V load that uses it.  Attention outputs at duplicate positions are thrown away by the gather
// (Algorithm 1, "Gather attention output"), and in a trie the representative tokens of a sequence are
// a SUFFIX of it (once a token opens a new node, so do all later ones), so only positions
// [first representative, len) are computed and their rows go straight into the compact attention
// output.  The work list (launch_attn_plan) cuts those positions into blocks of 32 queries, one per
// wavefront row slot.  Where a sequence has fewer blocks left than a workgroup has slots, the leftover
// blocks of consecutive sequences share a workgroup: all slots first walk the K/V tiles of the prefix
// the sequences have in common (read once, no causal boundary inside), then every slot in turn walks
// the remaining tiles of its own sequence while the other slots only help loading.  K/V tiles always
// start at multiples of 64 keys and a row meets them in increasing order, so every row's arithmetic
// is that of the full-layout mode and both modes give bit-identical rows.
#include "common.h"
#include "kernels.h"

namespace {

constexpr int HD = 128;
constexpr int BKV = 64;     // keys per tile
constexpr int ATT_THREADS = 256;
constexpr int TILE_SLOTS = BKV * 16;    // 16-byte slots of one K or V tile (16 KB)

typedef __attribute__((ext_vector_type(4))) short s16x4;

template <int N> __device__ __forceinline__ void att_wait_vmcnt() {
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}
// Asynchronous 16-byte-per-lane copy global -> LDS: lane L of the wavefront writes LDS bytes
// [lds_base + 16 L, +16); global address = uniform base + per-lane byte offset.
__device__ __forceinline__ void att_dma16(const void* base, uint32_t lane_off, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 ::"v"(lane_off), "s"(base), "s"(lds_base) : "memory");
}
__device__ __forceinline__ uint32_t att_lds_addr(const void* p) {
    return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) char*)p;
}

template <int DT, int HPB, bool FUSED, bool SPLIT>
__global__ __launch_bounds__(ATT_THREADS, SPLIT ? 1 : 2) void attention_mfma_kernel(const typename Op<DT>::T* __restrict__ qkv,
                                                                        const int32_t* __restrict__ cu, int N,
                                                                        int n_q_heads, int n_kv_heads, int n_qtiles,
                                                                        int n_pairs,
                                                                        typename Op<DT>::T* __restrict__ out,
                                                                        const int32_t* __restrict__ iscat,
                                                                        const int32_t* __restrict__ plan,
                                                                        AttnPlanLayout pl,
                                                                        int n_compact, int split_out) {
    typedef typename Op<DT>::T T;
    typedef typename Op<DT>::V8 V8;
    typedef typename Op<DT>::V4 V4;
    // [stage][key][16 chunks of 8 hd].  K: chunk ^= key & 15 (a fragment read walks 16 keys of one
    // chunk column).  V: chunk ^= (key & 3) << 2 (a transpose read walks 4 keys of one 64-byte column block).
    // SPLIT: q, k and v come as 16-bit (hi, lo) pairs (a row of the input is [q | k | v] hi, then [q | k | v] lo):
    // the tiles of both parts are staged, scores are K_hi Q_hi + K_hi Q_lo + K_lo Q_hi (the lo * lo term is below fp32
    // resolution) and the second product adds V_hi^T P^T and V_lo^T P^T.
    constexpr int NP = SPLIT ? 2 : 1;
    __shared__ uint4 Ks[2][NP][TILE_SLOTS];
    __shared__ uint4 Vs[2][NP][TILE_SLOTS];

    constexpr int BQ = 128 / HPB;                       // query rows per workgroup
    constexpr int WPH = 4 / HPB;                        // wavefronts per query head = 32-row slots per workgroup
    const int n_hg = n_q_heads / HPB;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 31, g = lane >> 5;
    const int wq = wave % WPH;                          // this wavefront's slot

    // ---- what this workgroup works on.  Per slot: sequence bounds and the first of its 32 query positions
    // (slot_len = 0: empty slot).  The K/V tiles come in phases: phase 0 = the first t_shared tiles, walked by all
    // slots through the map of slot 0's sequence; phase 1 + w = the further tiles of slot w's own sequence up to
    // its last query, walked by slot w alone.  The full-layout mode and single-sequence items are one phase 0.
    int hgroup;
    int slot_start[WPH], slot_len[WPH], slot_q[WPH];
    int t_shared, n_priv[WPH];
    if (!FUSED) {
        // Work item = (sequence, head group, query tile).  Workgroup ids are dealt round-robin to the 8 XCDs,
        // each with its own L2: id % 8 picks the XCD, and all query tiles of one (sequence, head group) - which
        // walk the same K/V rows - are given to the same XCD, consecutively.
        const int pair = ((int)blockIdx.x / 8 / n_qtiles) * 8 + (int)blockIdx.x % 8;    // (sequence, head group)
        if (pair >= n_pairs) return;
        const int seq = pair / n_hg;
        hgroup = pair % n_hg;
        const int qt = n_qtiles - 1 - ((int)blockIdx.x / 8) % n_qtiles;                  // heavy (late) tiles first
        // clamped so that a malformed cu_seqlens can never index outside the N rows
        int start = cu[seq], end = cu[seq + 1];
        start = start < 0 ? 0 : (start > N ? N : start);
        end = end < start ? start : (end > N ? N : end);
        if (qt * BQ >= end - start) return;
#pragma unroll
        for (int w = 0; w < WPH; ++w) {
            slot_start[w] = start;
            slot_len[w] = end - start;
            slot_q[w] = qt * BQ + 32 * w;
            n_priv[w] = 0;
        }
        const int last_q = (qt * BQ + BQ - 1) < (end - start - 1) ? (qt * BQ + BQ - 1) : (end - start - 1);
        t_shared = last_q / BKV + 1;
    } else {
        // Work index = XCD-major: each XCD gets a contiguous range of (head group, item), so the items that
        // share a KV head's prefix rows share an L2.
        const int n_items = plan[0];
        const long long total = (long long)n_items * n_hg;
        const long long per_xcd = (total + 7) / 8;
        const long long wi = (long long)((int)blockIdx.x % 8) * per_xcd + (int)blockIdx.x / 8;
        if ((int)blockIdx.x / 8 >= per_xcd || wi >= total) return;
        hgroup = (int)(wi / n_items);
        // last item first: the packed items, then every sequence's blocks from its last (most keys) to its first,
        // so that the workgroups still running when the grid drains are the light ones
        const int item = n_items - 1 - (int)(wi % n_items);
        const int ts = plan[pl.t_shared + item];
        int last_tile = -1;
#pragma unroll
        for (int w = 0; w < WPH; ++w) {
            const int sq = plan[pl.seq + 4 * item + w];
            int start = 0, end = 0;
            if (sq >= 0) {
                start = cu[sq]; end = cu[sq + 1];
                start = start < 0 ? 0 : (start > N ? N : start);
                end = end < start ? start : (end > N ? N : end);
            }
            int q0 = plan[pl.q + 4 * item + w];
            q0 = q0 < 0 ? 0 : q0;
            slot_start[w] = start;
            slot_len[w] = q0 < end - start ? end - start : 0;      // nothing to do: empty slot
            slot_q[w] = q0;
            const int lq = (q0 + 31) < (end - start - 1) ? (q0 + 31) : (end - start - 1);
            n_priv[w] = slot_len[w] > 0 ? lq / BKV + 1 : 0;          // for now: all tiles of the slot
            last_tile = n_priv[w] > last_tile ? n_priv[w] : last_tile;
        }
        if (last_tile <= 0) return;
        if (ts == 0x7FFFFFFF) {                                      // one sequence: a single phase with causal masks
            t_shared = last_tile;
#pragma unroll
            for (int w = 0; w < WPH; ++w) n_priv[w] = 0;
        } else {
            t_shared = slot_len[0] > 0 ? ts : 0;                     // phase 0 needs slot 0's map
#pragma unroll
            for (int w = 0; w < WPH; ++w) n_priv[w] = n_priv[w] > t_shared ? n_priv[w] - t_shared : 0;
        }
    }
    int n_tiles = t_shared;
#pragma unroll
    for (int w = 0; w < WPH; ++w) n_tiles += n_priv[w];

    const int start = slot_start[wq], len = slot_len[wq];     // this wavefront's own sequence
    const int q0w = slot_q[wq];
    const int group = n_q_heads / n_kv_heads;
    const int h = hgroup * HPB + wave / WPH;            // query head of this wavefront
    const int kvh = (hgroup * HPB) / group;             // one KV head per workgroup: HPB divides group
    const int dq = n_q_heads * HD, dkv = n_kv_heads * HD;
    const size_t row = ((size_t)dq + 2 * (size_t)dkv) * NP;     // elements of an input row (both parts)
    const size_t lo_off = (size_t)dq + 2 * (size_t)dkv;         // SPLIT: where the lo part of a row starts
    const uint32_t row_bytes = (uint32_t)(row * sizeof(T));
    // K/V base: the compact buffer (FUSED: rows come from the map) or, full layout, the rows of the one sequence
    const char* kbase = (const char*)(qkv + (FUSED ? (size_t)0 : (size_t)slot_start[0] * row) + dq + (size_t)kvh * HD);
    const char* vbase = kbase + (size_t)dkv * sizeof(T);
    auto compact_row = [&](int seq_start, int p) {              // clamped: a bad map can never leave the buffer
        int c = iscat[seq_start + p];
        c = c < 0 ? 0 : (c >= n_compact ? n_compact - 1 : c);
        return c;
    };
    // tile t of the workgroup's list -> (sequence whose keys it holds, first key); wave-uniform
    auto tile_of = [&](int t, int& t_start, int& t_len, int& kv0) {
        t_start = slot_start[0]; t_len = slot_len[0]; kv0 = t * BKV;
        int rest = t - t_shared;
#pragma unroll
        for (int w = 0; w < WPH; ++w) {
            if (rest >= 0 && rest < n_priv[w]) { t_start = slot_start[w]; t_len = slot_len[w]; kv0 = (t_shared + rest) * BKV; }
            rest -= n_priv[w];
        }
    };
    // which slot computes on tile t: -1 = all of them
    auto owner_of = [&](int t) {
        int own = -1, rest = t - t_shared;
#pragma unroll
        for (int w = 0; w < WPH; ++w) {
            if (rest >= 0 && rest < n_priv[w]) own = w;
            rest -= n_priv[w];
        }
        return own;
    };

    // ---- K/V tile loads: wavefront w fills tile rows [16 w, 16 w + 16) of K and of V, 4 rows (1 KB) per
    // instruction: lane L -> row 4 j + L / 16, LDS chunk L % 16, global chunk = LDS chunk ^ swizzle(row).
    // Rows past the end of the sequence are clamped (the causal mask hides them).
    const int lrow = lane >> 4, lpc = lane & 15;
    int krow[4];                                                // FUSED: compact rows of this lane's 4 keys of the tile to issue
    auto lookup_tile = [&](int t) {
        int ts, tl, kv0;
        tile_of(t, ts, tl, kv0);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int kr = kv0 + 16 * wave + 4 * j + lrow;
            kr = kr < tl ? kr : tl - 1;
            krow[j] = compact_row(ts, kr);
        }
    };
    auto issue_tile = [&](int t, int stage) {
        int ts, tl, kv0;
        tile_of(t, ts, tl, kv0);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int r = 16 * wave + 4 * j + lrow;             // tile row = key
            int kr = kv0 + r;
            kr = kr < tl ? kr : tl - 1;
            const uint32_t rb = (uint32_t)(FUSED ? krow[j] : kr) * row_bytes;
#pragma unroll
            for (int p = 0; p < NP; ++p) {
                att_dma16(kbase + p * lo_off * sizeof(T), rb + 16u * (uint32_t)(lpc ^ (r & 15)),
                          att_lds_addr(&Ks[stage][p][(16 * wave + 4 * j) * 16]));
                att_dma16(vbase + p * lo_off * sizeof(T), rb + 16u * (uint32_t)(lpc ^ ((r & 3) << 2)),
                          att_lds_addr(&Vs[stage][p][(16 * wave + 4 * j) * 16]));
            }
        }
    };
    const int wave_qmin = q0w, wave_qmax = q0w + 31;
    if (FUSED) lookup_tile(0);
    issue_tile(0, 0);
    if (FUSED && n_tiles > 1) lookup_tile(1);

    // ---- Q fragment (B operand of S^T = K Q^T): lane (n, g) holds Q[query n][16 ks + 8 g .. +8]
    const int qi = q0w + n;                             // query offset inside the sequence
    const int qi_c = qi < len ? qi : (len > 0 ? len - 1 : 0);
    V8 qf[NP][8];
    {
        const size_t qrow = FUSED ? (len > 0 ? (size_t)compact_row(start, qi_c) : (size_t)0) : (size_t)(start + qi_c);
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const uint4* qp = (const uint4*)(qkv + qrow * row + p * lo_off + (size_t)h * HD);
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                uint4 v = qp[ks * 2 + g];
                qf[p][ks] = *reinterpret_cast<V8*>(&v);
            }
        }
    }

    f32x16 o[4];
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int e = 0; e < 16; ++e) o[b][e] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;
    const float sc = 1.4426950408889634f / sqrtf((float)HD);     // log2(e) / sqrt(hd), applied inside the exponent

    // transpose-read addressing of V (see the header): 16-lane group = lane / 16 -> g = group / 2,
    // 16-column half = group % 2; inside the group lane i = 4 e + a reads key e, columns 4 a .. 4 a + 3.
    const int tr_e = (lane >> 2) & 3, tr_a = lane & 3, tr_half = (lane >> 4) & 1;
    // byte offset inside a V tile of (key 4 g + tr_e [+ 16 kk + 8 second], columns 32 b + 16 half + 4 a):
    //   key * 256 + ((chunk ^ (tr_e << 2)) << 4) + (a & 1) * 8   with chunk = 4 b + 2 half + a / 2
    const uint32_t tr_key0 = (uint32_t)(4 * g + tr_e) * 256u + (uint32_t)(tr_a & 1) * 8u;
    const int tr_chunk0 = 2 * tr_half + (tr_a >> 1);

    for (int t = 0; t < n_tiles; ++t) {
        const int st = t & 1;
        att_wait_vmcnt<0>();                // this wavefront's share of tile t has landed
        __syncthreads();                    // everybody's has; everybody is done with tile t-1
        if (t + 1 < n_tiles) issue_tile(t + 1, st ^ 1);
        if (FUSED && t + 2 < n_tiles) lookup_tile(t + 2);   // rows of tile t+2, waited for with tile t+1
        int kv0 = t * BKV;
        if (FUSED) {
            int ts_, tl_;
            tile_of(t, ts_, tl_, kv0);
            const int own = owner_of(t);
            if (len <= 0 || (own >= 0 && own != wq)) continue;      // empty slot, or another slot's own tiles
        }
        if (kv0 > wave_qmax) continue;      // whole tile is in this wavefront's future

        // ---- S^T = K Q^T : two 32-key blocks x 8 k-steps.  The K fragments are read from LDS four MFMAs
        // ahead of their use (the scheduling barriers pin that order), so LDS latency hides behind the
        // matrix pipe.  MFMA t: key block t & 1, k-step t >> 1.
        f32x16 s[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int e = 0; e < 16; ++e) s[kb][e] = 0.f;
        {
            // terms: K_hi Q_hi [, K_hi Q_lo, K_lo Q_hi]; MFMA u: term u >> 4, key block u & 1, k-step (u & 15) >> 1
            constexpr int NS_ = (SPLIT ? 3 : 1) * 16;
            uint4 kf[16];
            auto read_k = [&](int u) {
                const int uu = u & 15, key = (uu & 1) * 32 + n;
                kf[uu] = Ks[st][(u >> 4) == 2 ? NP - 1 : 0][key * 16 + (((uu >> 1) * 2 + g) ^ (key & 15))];
            };
#pragma unroll
            for (int u = 0; u < 4; ++u) read_k(u);
#pragma unroll
            for (int u = 0; u < NS_; ++u) {
                if (u + 4 < NS_) read_k(u + 4 < NS_ ? u + 4 : 0);
                s[u & 1] = Op<DT>::mfma(*reinterpret_cast<V8*>(&kf[u & 15]), qf[(u >> 4) == 1 ? NP - 1 : 0][(u & 15) >> 1], s[u & 1]);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        // V^T fragments of the second product, MFMA u: k-step u >> 2 (16 keys), hd block u & 3.  The first
        // four are requested now and arrive during the softmax.
        // (SPLIT: u >> 4 picks the part of V; the ring of 16 fragment registers is indexed by u & 15)
        constexpr int NV_ = NP * 16;
        s16x4 vlo[16], vhi[16];
        auto read_v = [&](int u) {
            const char* vt = (const char*)&Vs[st][u >> 4][0];
            const int kk = (u & 15) >> 2, b = u & 3;
            const uint32_t off = tr_key0 + (uint32_t)kk * 4096u + (uint32_t)(((4 * b + tr_chunk0) ^ (tr_e << 2)) << 4);
            vlo[u & 15] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(vt + off));
            vhi[u & 15] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(vt + off + 2048u));
        };
#pragma unroll
        for (int u = 0; u < 4; ++u) read_v(u);
        __builtin_amdgcn_sched_barrier(0);

        // ---- causal mask on diagonal tiles (register e of block kb is key kv0 + 32 kb + 8 (e/4) + 4 g + e%4),
        // running maximum of the raw scores, p = 2^(s c - m c) with one fma + one v_exp per element
        if ((kv0 + BKV - 1) > wave_qmin) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int kj = kv0 + kb * 32 + 8 * (e >> 2) + 4 * g + (e & 3);
                    if (kj > qi_c) s[kb][e] = -INFINITY;
                }
        }
        float tmax = s[0][0];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int e = 0; e < 16; ++e) tmax = fmaxf(tmax, s[kb][e]);
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
        const float m_new = fmaxf(m_run, tmax);       // finite: tile 0 always holds key 0 <= query
        const float neg_mc = -m_new * sc;
        float psum = 0.f;
        V8 pf[4];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const float p = __builtin_amdgcn_exp2f(fmaf(s[kb][e], sc, neg_mc));
                psum += p;
                pf[kb * 2 + (e >> 3)][e & 7] = (T)p;
            }
        // rescale the running sums only when some query of the wavefront saw a new maximum
        if (__any(m_new != m_run)) {
            const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * sc);     // 0 on the first tile (m_run = -inf)
            l_run *= alpha;
#pragma unroll
            for (int b = 0; b < 4; ++b)
#pragma unroll
                for (int e = 0; e < 16; ++e) o[b][e] *= alpha;
        }
        l_run += psum;
        m_run = m_new;

        // ---- O^T += V^T P^T : 4 k-steps of 16 keys x 4 hd blocks, V^T fragments read four MFMAs ahead.
        // Key order inside a k-step: the lo read holds keys 16 kk + 4 g + 0..3, the hi read 16 kk + 8 + 4 g + 0..3,
        // which is the order the P^T registers of k-step kk are in.
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < NV_; ++u) {
            if (u + 4 < NV_) read_v(u + 4 < NV_ ? u + 4 : 0);
            union { struct { s16x4 lo, hi; } p; V8 v; } cvt;
            cvt.p.lo = vlo[u & 15];
            cvt.p.hi = vhi[u & 15];
            o[u & 3] = Op<DT>::mfma(cvt.v, pf[(u & 15) >> 2], o[u & 3]);
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    // ---- normalise and store: register e of block b is hd = 32 b + 8 (e/4) + 4 g + e%4.
    // split_out: the row is [hi | lo] with hi = T(o) and lo = T(o - hi), for an output projection over the doubled K.
    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    if (qi < len) {
        const float inv = 1.0f / l_tot;
        const size_t orow = FUSED ? (size_t)compact_row(start, qi) : (size_t)(start + qi);
        T* op = out + orow * (size_t)(split_out ? 2 * dq : dq) + (size_t)h * HD;
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                V4 v, lo;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float x = o[b][q4 * 4 + j] * inv;
                    v[j] = (T)x;
                    lo[j] = (T)(x - (float)v[j]);
                }
                *reinterpret_cast<V4*>(op + b * 32 + q4 * 8 + g * 4) = v;
                if (split_out) *reinterpret_cast<V4*>(op + dq + b * 32 + q4 * 8 + g * 4) = lo;
            }
    }
}

}  // namespace

static int launch_attention_any(const void* qkv, const int32_t* cu, int B, int N, int max_seqlen, int n_q_heads,
                                int n_kv_heads, int hd, void* out, int op_dtype, const int32_t* iscat,
                                const int32_t* plan, int n_compact, int split_out, int split_in, hipStream_t stream) {
    const bool fused = iscat != nullptr;
    if (N <= 0 || B <= 0) return RADIX_OK;
    if (hd != HD) return RADIX_ERR_UNSUPPORTED;
    if (!fused && max_seqlen <= 0) return RADIX_ERR_BAD_SIZE;
    if (op_dtype != RADIX_BF16 && op_dtype != RADIX_F16) return RADIX_ERR_UNSUPPORTED;
    if ((((uintptr_t)qkv | (uintptr_t)out) & 15) != 0) return RADIX_ERR_MISALIGNED;
    if (fused && (plan == nullptr || n_compact <= 0)) return RADIX_ERR_BAD_SIZE;
    const int group = n_q_heads / n_kv_heads;
    const int hpb = (group % 4 == 0) ? 4 : (group % 2 == 0 ? 2 : 1);    // query heads per workgroup
    const AttnPlanLayout pl = attn_plan_layout((size_t)N, (size_t)B);
    int n_qtiles = 0, n_pairs = 0;
    long long n_blocks;
    if (fused) {
        // The item count is known on the device only.  Its bound: every sequence cuts its R_s representative rows
        // (sum R_s = n_compact) into ceil(R_s / 32) blocks, `slots` blocks make an item, the packed items round
        // up once.  Workgroups past the real count leave at once (they still cost a launch each, hence the
        // tight bound).
        const int slots = 4 / hpb;
        long long items = ((long long)n_compact / 32 + B + slots - 1) / slots + 1;
        if (items > pl.max_items) items = pl.max_items;
        n_blocks = (items * (n_q_heads / hpb) + 7) / 8 * 8;
    } else {
        n_qtiles = ceil_div(max_seqlen, 128 / hpb);
        n_pairs = (n_q_heads / hpb) * B;
        n_blocks = (long long)ceil_div(n_pairs, 8) * 8 * n_qtiles;
    }
    if (n_blocks > 0x7FFFFFFFLL) return RADIX_ERR_UNSUPPORTED;
    // per-lane 32-bit byte offsets: inside one sequence's K/V rows, or (fused) inside the compact buffer
    const long long span_rows = fused ? (long long)n_compact : (long long)max_seqlen;
    if (span_rows * (n_q_heads + 2 * n_kv_heads) * HD * 2 * (split_in ? 2 : 1) >= (1LL << 32)) return RADIX_ERR_UNSUPPORTED;
    const dim3 grid((unsigned)n_blocks), block(ATT_THREADS);
#define RADIX_ATT(DT, HPB, F, S)                                                                                   \
    hipLaunchKernelGGL((attention_mfma_kernel<DT, HPB, F, S>), grid, block, 0, stream, (const Op<DT>::T*)qkv, cu,  \
                       N, n_q_heads, n_kv_heads, n_qtiles, n_pairs, (Op<DT>::T*)out, iscat, plan, pl, n_compact,   \
                       split_out)
#define RADIX_ATT_H(DT, F, S)                                                                                      \
    do {                                                                                                           \
        if (hpb == 4) RADIX_ATT(DT, 4, F, S); else if (hpb == 2) RADIX_ATT(DT, 2, F, S); else RADIX_ATT(DT, 1, F, S); \
    } while (0)
#define RADIX_ATT_S(DT, F)                                                                                         \
    do {                                                                                                           \
        if (split_in) RADIX_ATT_H(DT, F, true); else RADIX_ATT_H(DT, F, false);                                    \
    } while (0)
    if (op_dtype == RADIX_BF16) {
        if (fused) RADIX_ATT_S(RADIX_BF16, true); else RADIX_ATT_S(RADIX_BF16, false);
    } else {
        if (fused) RADIX_ATT_S(RADIX_F16, true); else RADIX_ATT_S(RADIX_F16, false);
    }
#undef RADIX_ATT_S
#undef RADIX_ATT_H
#undef RADIX_ATT
    return RADIX_OK;
}

int launch_attention_mfma(const void* qkv, const int32_t* cu, int B, int N, int max_seqlen, int n_q_heads,
                          int n_kv_heads, int hd, void* out, int op_dtype, hipStream_t stream, int split_out,
                          int split_in) {
    return launch_attention_any(qkv, cu, B, N, max_seqlen, n_q_heads, n_kv_heads, hd, out, op_dtype, nullptr, nullptr,
                                0, split_out, split_in, stream);
}

int launch_attention_mfma_fused(const void* qkv_c, const int32_t* cu, const int32_t* I_scatter,
                                const int32_t* plan, int B, int N, int n_compact, int n_q_heads,
                                int n_kv_heads, int hd, void* out_c, int op_dtype, hipStream_t stream, int split_out,
                                int split_in) {
    if (I_scatter == nullptr) return RADIX_ERR_BAD_SIZE;
    return launch_attention_any(qkv_c, cu, B, N, 0, n_q_heads, n_kv_heads, hd, out_c, op_dtype, I_scatter,
                                plan, n_compact, split_out, split_in, stream);
}
