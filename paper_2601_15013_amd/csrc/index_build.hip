// GPU builder of the prefix-trie index maps I_scatter / I_gather.
//
// What is computed is fixed by the paper (Approach, "Trie Construction" and "Gather and Scatter
// Kernels"; appendix Algorithm 2 with its "Index semantics"): nodes are path-specific, compact
// ids are handed out in order of first occurrence.  How it is computed here is not the
// sequential insertion of Algorithm 2 but a level-synchronous, "follow the leader" scheme:
//
//   * Every sequence s follows a leader: the lowest-numbered sequence known to share s's path
//     so far.  All sequences start by following the first non-empty sequence.
//   * One round = one trie branching level on each follower's path.  A wavefront compares the
//     follower with its leader 256 tokens at a time (coalesced loads + ballot) until the first
//     (token, position) mismatch m.  Positions below m are duplicates of the leader's nodes.
//   * Followers that leave the same leader at the same depth with the same (token, position)
//     key enter the same child node.  They are grouped by an exact open-addressing table
//     (keys are compared in full, the hash only picks the probe start); the lowest-numbered
//     member becomes the leader of the new node and all its later positions are new nodes,
//     the others follow it in the next round.
//   * A sequence becomes a leader at most once, so there are at most (deepest branching
//     chain) rounds, and every position is compared exactly once: O(N) work in total.
//   * New nodes of sequence s are its positions >= b_s (the depth where it became a leader),
//     a contiguous tail, so compact ids are cbase_s + (p - b_s) with cbase the exclusive
//     wavefront scan of (len_s - b_s) over sequences: exactly first-occurrence order.
//
// The chain phase runs in one 1024-thread workgroup (it is latency-bound bookkeeping over B
// sequences; the data is 4N bytes); the final map write-out is a chip-wide kernel over tokens.
#include <mutex>

#include "common.h"
#include "kernels.h"

namespace {

constexpr int IDX_THREADS = 1024;
constexpr int IDX_WAVES = IDX_THREADS / RADIX_WAVE;
constexpr int LCP_UNROLL = 4;

__device__ __forceinline__ int ld_agent(const int* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ uint32_t key_hash(int l, int m, int t, int pp) {
    uint64_t x = (((uint64_t)(uint32_t)l << 32) | (uint32_t)m) * 0x9E3779B97F4A7C15ull;
    x ^= ((uint64_t)(uint32_t)pp << 32) | (uint32_t)t;
    x ^= x >> 29;
    x *= 0xBF58476D1CE4E5B9ull;
    x ^= x >> 32;
    return (uint32_t)x;
}

__global__ __launch_bounds__(IDX_THREADS) void index_chain_kernel(
    const int32_t* __restrict__ tok, const int32_t* __restrict__ pos, const int32_t* __restrict__ cu,
    int B, int N, int32_t* __restrict__ lead, int32_t* hdr, int32_t* ldr, int32_t* dep, int32_t* bdep,
    int32_t* mis, int32_t* myslot, int32_t* cbase, int32_t* slot_owner, int32_t* slot_min, int H,
    int32_t* n_compact_dev) {
    __shared__ int sh_first;
    __shared__ int sh_wave_tot[IDX_WAVES];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    // every call starts with a clean status word
    if (tid == 0) hdr[0] = 0;

    // ---- validate cu_seqlens before anything is dereferenced through it
    int bad = 0;
    for (int i = tid; i <= B; i += IDX_THREADS) {
        int c = cu[i];
        if (c < 0 || c > N) bad = 1;
        if (i == 0 && c != 0) bad = 1;
        if (i == B && c != N) bad = 1;
        if (i < B && cu[i + 1] < c) bad = 1;
    }
    bad = __syncthreads_or(bad);
    if (bad) {
        if (tid == 0) {
            set_status(hdr, RADIX_ERR_BAD_CU_SEQLENS);
            hdr[1] = 0;
            *n_compact_dev = 0;
        }
        return;
    }

    // ---- initial state: everybody follows the first non-empty sequence
    if (tid == 0) sh_first = B;
    __syncthreads();
    for (int s = tid; s < B; s += IDX_THREADS)
        if (cu[s + 1] - cu[s] > 0) atomicMin(&sh_first, s);
    __syncthreads();
    const int s0 = sh_first;
    for (int s = tid; s < B; s += IDX_THREADS) {
        int len = cu[s + 1] - cu[s];
        mis[s] = -1;
        if (len == 0 || s == s0) {
            bdep[s] = 0;      // leader from depth 0 (or empty)
            ldr[s] = -1;
        } else {
            bdep[s] = -1;     // -1 marks an active follower
            ldr[s] = s0;
            dep[s] = 0;
        }
    }
    for (int h = tid; h < H; h += IDX_THREADS) {
        slot_owner[h] = -1;
        slot_min[h] = 0x7FFFFFFF;
    }
    __syncthreads();

    // ---- rounds.  Each active follower's matched depth grows by >= 1 per round, so the loop
    // ends after at most (longest sequence + 1) rounds; N + 2 is a hard upper bound.
    for (int round = 0; round < N + 2; ++round) {
        // step 1: longest common prefix with the leader, one wavefront per follower
        int any = 0;
        for (int s = wave; s < B; s += IDX_WAVES) {
            if (bdep[s] != -1) continue;
            any = 1;
            const int l = ldr[s], st = dep[s];
            const int bs = cu[s], bl = cu[l];
            const int len_s = cu[s + 1] - bs, len_l = cu[l + 1] - bl;
            const int lim = len_s < len_l ? len_s : len_l;
            int m = lim;
            for (int p0 = st; p0 < lim; p0 += 64 * LCP_UNROLL) {
                int neq[LCP_UNROLL];
#pragma unroll
                for (int u = 0; u < LCP_UNROLL; ++u) {
                    int p = p0 + u * 64 + lane;
                    bool valid = p < lim;
                    int a = valid ? tok[bs + p] : 0;
                    int b = valid ? tok[bl + p] : 1;
                    int d = (a != b);
                    if (pos != nullptr && valid) d |= (pos[bs + p] != pos[bl + p]);
                    neq[u] = d;
                }
                bool stop = false;
#pragma unroll
                for (int u = 0; u < LCP_UNROLL; ++u) {
                    if (stop) continue;
                    int p = p0 + u * 64 + lane;
                    unsigned long long mask = __ballot(neq[u]);
                    if (mask == 0ull) {
                        lead[bs + p] = l;
                    } else {
                        int first = __ffsll((long long)mask) - 1;
                        if (lane < first) lead[bs + p] = l;
                        m = p0 + u * 64 + first;
                        stop = true;
                    }
                }
                if (stop) break;
            }
            if (lane == 0) {
                if (m == len_s) {       // s ran out while still equal to its leader: no new node
                    bdep[s] = len_s;
                    ldr[s] = -1;
                } else {
                    mis[s] = m;         // s leaves its leader at depth m
                }
            }
        }
        if (!__syncthreads_or(any)) break;

        // step 2: group the leavers by (leader, depth, token, position) - exact comparison
        for (int s = tid; s < B; s += IDX_THREADS) {
            if (bdep[s] != -1) continue;
            const int l = ldr[s], m = mis[s];
            const int t = tok[cu[s] + m];
            const int pp = pos ? pos[cu[s] + m] : m;
            uint32_t h = key_hash(l, m, t, pp) & (uint32_t)(H - 1);
            for (int probe = 0; probe < H; ++probe) {
                int o = ld_agent(&slot_owner[h]);
                if (o == -1) {
                    o = atomicCAS(&slot_owner[h], -1, s);
                    if (o == -1) o = s;
                }
                if (o == s) break;
                if (ldr[o] == l && mis[o] == m && tok[cu[o] + m] == t && (pos ? pos[cu[o] + m] : m) == pp) break;
                h = (h + 1) & (uint32_t)(H - 1);
            }
            atomicMin(&slot_min[h], s);
            myslot[s] = (int)h;
        }
        __syncthreads();

        // step 3: lowest member leads the new node, the others follow it
        for (int s = tid; s < B; s += IDX_THREADS) {
            if (bdep[s] != -1) continue;
            const int c = ld_agent(&slot_min[myslot[s]]);
            const int m = mis[s];
            if (c == s) {
                bdep[s] = m;
                ldr[s] = -1;
            } else {
                ldr[s] = c;
                dep[s] = m;
            }
        }
        __syncthreads();
        for (int s = tid; s < B; s += IDX_THREADS) {
            if (mis[s] < 0) continue;
            const int h = myslot[s];
            slot_owner[h] = -1;
            slot_min[h] = 0x7FFFFFFF;
            mis[s] = -1;
        }
        __syncthreads();
    }

    // ---- compact-id base of every sequence: exclusive scan of its count of new nodes
    int running = 0;
    for (int base = 0; base < B; base += IDX_THREADS) {
        const int s = base + tid;
        int cnt = 0;
        if (s < B) {
            int b = bdep[s];
            int len = cu[s + 1] - cu[s];
            if (b < 0) {            // cannot happen (loop bound); keep the maps well-formed anyway
                b = len;
                bdep[s] = len;
                set_status(hdr, RADIX_ERR_BAD_SIZE);
            }
            cnt = len - b;
        }
        int incl = cnt;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            int v = __shfl_up(incl, o, 64);
            if (lane >= o) incl += v;
        }
        if (lane == 63) sh_wave_tot[wave] = incl;
        __syncthreads();
        int before = 0, total = 0;
#pragma unroll
        for (int w = 0; w < IDX_WAVES; ++w) {
            int v = sh_wave_tot[w];
            if (w < wave) before += v;
            total += v;
        }
        if (s < B) cbase[s] = running + before + incl - cnt;
        running += total;
        __syncthreads();
    }
    if (tid == 0) {
        *n_compact_dev = running;
        hdr[1] = running;
    }
}

// One thread per original position: turn (leader sequence, offset) into compact ids.
__global__ __launch_bounds__(256) void index_finalize_kernel(
    const int32_t* __restrict__ tok, const int32_t* __restrict__ pos, const int32_t* __restrict__ cu,
    int B, int N, int32_t* __restrict__ I_scatter /* holds leader ids of duplicate positions */,
    int32_t* __restrict__ I_gather, int32_t* hdr, const int32_t* __restrict__ bdep,
    const int32_t* __restrict__ cbase) {
    if (ld_agent(&hdr[0]) == RADIX_ERR_BAD_CU_SEQLENS) return;
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= N) return;
    // sequence of j: smallest s with cu[s+1] > j
    int lo = 0, hi = B - 1;
    while (lo < hi) {
        int mid = (lo + hi) >> 1;
        if (cu[mid + 1] > j) hi = mid; else lo = mid + 1;
    }
    const int s = lo;
    const int p = j - cu[s];
    if (tok[j] < 0 || (pos != nullptr && pos[j] < 0)) set_status(hdr, RADIX_ERR_BAD_TOKEN);
    const int b = bdep[s];
    if (p >= b) {
        const int c = cbase[s] + (p - b);
        I_scatter[j] = c;
        I_gather[c] = j;
    } else {
        const int l = I_scatter[j];
        I_scatter[j] = cbase[l] + (p - bdep[l]);
    }
}

int next_pow2(int x) {
    int h = 64;
    while (h < x) h <<= 1;
    return h;
}

}  // namespace

size_t radix_index_ws_bytes(int B) {
    size_t H = (size_t)next_pow2(2 * (B > 0 ? B : 1));
    return RADIX_WS_HEADER_BYTES + align_up(((size_t)6 * (size_t)(B > 0 ? B : 1) + 2 * H) * sizeof(int32_t), 256);
}

extern "C" int radix_index_workspace_bytes(int32_t max_B, size_t* bytes_out) {
    if (!bytes_out) return RADIX_ERR_NULL_POINTER;
    if (max_B < 0) return RADIX_ERR_BAD_SIZE;
    *bytes_out = radix_index_ws_bytes(max_B);
    return RADIX_OK;
}

namespace {

int build_index_impl(const int32_t* tok, const int32_t* pos, const int32_t* cu_seqlens, int32_t B, int32_t N,
                     int32_t* I_scatter, int32_t* I_gather, int32_t* n_compact_dev, int32_t* n_compact_host,
                     void* ws, hipStream_t stream) {
    int32_t* hdr = (int32_t*)ws;
    int32_t* base = (int32_t*)((char*)ws + RADIX_WS_HEADER_BYTES);
    const size_t Bn = (size_t)(B > 0 ? B : 1);
    const int H = next_pow2(2 * (int)Bn);
    int32_t* ldr = base;
    int32_t* dep = ldr + Bn;
    int32_t* bdep = dep + Bn;
    int32_t* mis = bdep + Bn;
    int32_t* myslot = mis + Bn;
    int32_t* cbase = myslot + Bn;
    int32_t* slot_owner = cbase + Bn;
    int32_t* slot_min = slot_owner + H;

    // the chain kernel initialises every word of builder state it reads (status word, per-sequence arrays, both
    // slot tables), so the buffer may hold anything when the call starts
    hipLaunchKernelGGL(index_chain_kernel, dim3(1), dim3(IDX_THREADS), 0, stream, tok, pos, cu_seqlens, B, N,
                       I_scatter, hdr, ldr, dep, bdep, mis, myslot, cbase, slot_owner, slot_min, H, n_compact_dev);
    if (N > 0) {
        hipLaunchKernelGGL(index_finalize_kernel, dim3(ceil_div(N, 256)), dim3(256), 0, stream, tok, pos,
                           cu_seqlens, B, N, I_scatter, I_gather, hdr, bdep, cbase);
    }
    HIP_TRY(hipGetLastError());
    if (n_compact_host) {
        int32_t h2[2] = {0, 0};
        HIP_TRY(hipMemcpyAsync(h2, hdr, sizeof(h2), hipMemcpyDeviceToHost, stream));
        HIP_TRY(hipStreamSynchronize(stream));
        *n_compact_host = h2[1];
        if (h2[0] != 0) return h2[0];
    }
    return RADIX_OK;
}

int check_index_args(const int32_t* tok, const int32_t* cu_seqlens, int32_t B, int32_t N, const int32_t* I_scatter,
                     const int32_t* I_gather, const int32_t* n_compact_dev) {
    if (B < 0 || N < 0) return RADIX_ERR_BAD_SIZE;
    if (B > (1 << 28)) return RADIX_ERR_BAD_SIZE;
    if (!cu_seqlens || !n_compact_dev) return RADIX_ERR_NULL_POINTER;
    if (N > 0 && (!tok || !I_scatter || !I_gather)) return RADIX_ERR_NULL_POINTER;
    if (N > 0 && B == 0) return RADIX_ERR_BAD_SIZE;
    return RADIX_OK;
}

}  // namespace

extern "C" int radix_build_index(const int32_t* tok, const int32_t* pos, const int32_t* cu_seqlens,
                                 int32_t B, int32_t N, int32_t* I_scatter, int32_t* I_gather,
                                 int32_t* n_compact_dev, int32_t* n_compact_host,
                                 void* ws, size_t ws_bytes, void* stream) {
    const int rc = check_index_args(tok, cu_seqlens, B, N, I_scatter, I_gather, n_compact_dev);
    if (rc != RADIX_OK) return rc;
    if (!ws) return RADIX_ERR_NULL_POINTER;
    if (((uintptr_t)ws & 255) != 0) return RADIX_ERR_MISALIGNED;
    if (ws_bytes < radix_index_ws_bytes(B)) return RADIX_ERR_WORKSPACE_TOO_SMALL;
    return build_index_impl(tok, pos, cu_seqlens, B, N, I_scatter, I_gather, n_compact_dev, n_compact_host, ws,
                            (hipStream_t)stream);
}

// ---- the same builder for callers that cannot allocate: its state lives in a static device array
// instead of a caller-provided workspace.  Every GPU the library runs on holds its own copy of the
// array at its own address; host code only ever uses the address hipGetSymbolAddress reports for
// the current device (the array's name is not a device address on the host side).
namespace {

constexpr size_t STATIC_INDEX_BYTES =
    RADIX_WS_HEADER_BYTES + ((size_t)6 * RADIX_STATIC_INDEX_MAX_B + 2 * (size_t)(2 * RADIX_STATIC_INDEX_MAX_B)) * sizeof(int32_t);
static_assert((RADIX_STATIC_INDEX_MAX_B & (RADIX_STATIC_INDEX_MAX_B - 1)) == 0 && RADIX_STATIC_INDEX_MAX_B >= 64,
              "the slot tables hold next_pow2(2 B) entries each");
static __device__ __align__(256) unsigned char scratch[STATIC_INDEX_BYTES];

constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[MAX_DEVICES] = {};

// address of `scratch` on the current device, looked up once per device
int static_scratch(void** out) {
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEVICES) return RADIX_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return RADIX_ERR_HIP;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return RADIX_OK;
}

}  // namespace

extern "C" int radix_build_index_static(const int32_t* tok, const int32_t* pos, const int32_t* cu_seqlens,
                                        int32_t B, int32_t N, int32_t* I_scatter, int32_t* I_gather,
                                        int32_t* n_compact_dev, int32_t* n_compact_host, void* stream) {
    int rc = check_index_args(tok, cu_seqlens, B, N, I_scatter, I_gather, n_compact_dev);
    if (rc != RADIX_OK) return rc;
    if (B > RADIX_STATIC_INDEX_MAX_B) return RADIX_ERR_STATIC_LIMIT;
    void* ws = nullptr;
    if ((rc = static_scratch(&ws)) != RADIX_OK) return rc;
    return build_index_impl(tok, pos, cu_seqlens, B, N, I_scatter, I_gather, n_compact_dev, n_compact_host, ws,
                            (hipStream_t)stream);
}
