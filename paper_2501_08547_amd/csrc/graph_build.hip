// Computation-graph construction for one batch, on the device, in integers only.
//
// Steps (paper passages): candidates = distinct training endpoints of the request's edges
// and the number of query edges at each (Sec. 5.2.1); recompute targets = the best
// floor(gamma |R|) candidates by query-edge ratio (Sec. 5.2.2, budget of Eq. 2); rows of the
// inner layers = queries and targets, each target row holding every edge that ends at it,
// from the base graph and from the request (Sec. 6.1).  The output is the canonical tagged
// CSR described in omega_srpe.h plus a work list that cuts long rows into parts.
//
// How: no global sort.  Query-edge counts are integer atomics into per-node / per-query
// counters; a bitmap over node ids turns "touched" into the ascending candidate list with one
// prefix sum; the recompute set is found by a most-significant-digit radix *select* on exact
// 64-bit ratio keys (ties resolved by a prefix sum in id order); edges are dropped into their
// rows with atomic cursors and every row is then sorted on its own (short ones by one wavefront,
// longer ones by a tiled rank sort), which makes the result independent of atomic ordering.
// Counters that many threads hit are kept in LDS per block and flushed once, or updated once per
// wavefront: global atomics on one address serialise at roughly 13 ns each on this part.  The flushed
// counters and histogram bins are packed, not spread one per cache line: spreading them was measured
// slower (the kernels that read and clear them then touch a line per counter).
// Prefix sums have no kernels of their own where it can be avoided: a producer leaves the total of every chunk
// of 64 (or block of 1,024) items and the consumer's block adds up the totals before its own (a few thousand
// values at most, L2 hits) and scans its own chunk locally.
// The sizes reach the host through pinned memory that the last kernel of the first half writes; waiting for
// that kernel is the only host synchronisation of a batch.
#include "internal.h"

#include <chrono>
#include <cstddef>
#include <cstring>
#include <type_traits>

namespace {

constexpr int TPB = 256;
constexpr int SEL_BITS = 13;                 // digit width of the radix select
constexpr int SEL_BINS = 1 << SEL_BITS;
constexpr int SEL_ITEMS = 4;                 // keys per thread in a select pass (1024 threads)
constexpr int SORT_WAVE_MAX = 64;            // segment lengths handled by one wavefront
constexpr int SORT_MED_MAX = 4096;           // ... by a 256-thread block; longer ones by a 1024-thread block
constexpr int SORT_KEYS = 16;                // keys a thread of the block sorts holds in registers
constexpr int EDGE_BLOCK = 1024;             // threads of the edge-list kernels (256 for small requests: they read blockDim)
// Request edges per thread in those kernels: 1, 2 or 4, the smallest that keeps the launch at 256 blocks or
// fewer.  The kernels are chains of dependent atomics, so they want many blocks; each block also zeroes and
// flushes n_query LDS counters, so they do not want more blocks than compute units.  (One fixed value of 4
// left `large`, 0.18 M request edges, with 44 blocks: graph construction 22 us slower.)
inline int edge_items(int64_t n_e) {
    return n_e <= 256 * (int64_t)EDGE_BLOCK ? 1 : n_e <= 512 * (int64_t)EDGE_BLOCK ? 2 : 4;
}
constexpr int LDS_QUERY_MAX = 16384;         // largest batch whose per-query counters fit in LDS
constexpr int SUM_BLOCK = 1024;              // items per block total of the flag and row prefix sums
constexpr int SELECT_ONE_BLOCK_MAX = 65536;  // up to this many candidates the whole radix select runs in one block
constexpr int ORDER_PHASES = 8;              // regions of a table the inner layers' work items are grouped by
__host__ __device__ inline int phase_first(int f, int np) { return (f * np + ORDER_PHASES - 1) / ORDER_PHASES; }   // ceil(f np / P)
constexpr int64_t TWO_LEVEL_WORDS = 262144;  // bitmaps longer than this many words (8.4 M nodes) get a second level (see k_list_words)

struct SelState {
    unsigned long long prefix;   // digits chosen so far (value of key >> lo of the last pass)
    long long k_rem;             // how many still to take inside the current prefix bucket
    long long k_take;            // floor(gamma |R|)
    long long n_list;            // keys that matched the first digit (k_select_compact)
    int take_none;
    int pad;
};

struct DevState {                // one allocation, cleared with one memset per build
    BuildCounts counts;
    SelState sel;
    long long n_touched_words;   // two-level bitmap: words of the node bitmap that hold a candidate
    // work items per region of the table (see fill_parts_body), and the cursors that hand out places inside a
    // region; one counter per 64 bytes
    long long phase_total[ORDER_PHASES * 8];
    long long phase_rank[ORDER_PHASES * 8];
    unsigned int hist[SEL_BINS];
};

inline unsigned grid_for(int64_t n, int64_t per_block = TPB) {
    const int64_t g = (n + per_block - 1) / per_block;
    return (unsigned)(g > 0 ? g : 1);
}

__device__ inline int64_t gtid() { return (int64_t)blockIdx.x * blockDim.x + threadIdx.x; }

__device__ inline int64_t base_deg(const int64_t* __restrict__ indptr, int32_t u) {
    return indptr[(int64_t)u + 1] - indptr[u];
}

// One atomic per wavefront: the lanes with pred == true get consecutive slots of *counter.
// Must be called by all lanes of the wavefront.
__device__ inline int64_t wave_append(bool pred, long long* counter) {
    const unsigned long long mask = __ballot(pred);
    const int lane = threadIdx.x & 63;
    const int leader = mask ? __ffsll((long long)mask) - 1 : 0;
    unsigned long long base = 0;
    if (lane == leader && mask) base = atomicAdd((unsigned long long*)counter, (unsigned long long)__popcll(mask));
    base = __shfl(base, leader);
    return (int64_t)base + __popcll(mask & ((1ull << lane) - 1ull));
}

// exclusive prefix sum of up to 1024 values held one per thread; every thread gets the block total
__device__ inline int64_t block_excl_scan(int64_t v, int64_t* total, int64_t* wave_tot /* [16] shared */) {
    const int lane = threadIdx.x & 63, wid = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
    int64_t x = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int64_t y = __shfl_up(x, off);
        if (lane >= off) x += y;
    }
    if (lane == 63) wave_tot[wid] = x;
    __syncthreads();
    int64_t before = 0, all = 0;
    for (int w = 0; w < nw; ++w) {
        const int64_t t = wave_tot[w];
        if (w < wid) before += t;
        all += t;
    }
    __syncthreads();
    *total = all;
    return before + x - v;
}

__device__ inline int64_t wave_sum_i64(int64_t x) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off);
    return x;
}

// sum of tot[0 .. n) computed by all threads of the block together; every thread gets it.  sh: 16 values of LDS.
template <typename T>
__device__ inline int64_t block_sum_of(const T* __restrict__ tot, int64_t n, int64_t* sh) {
    int64_t s = 0;
    for (int64_t i = threadIdx.x; i < n; i += blockDim.x) s += (int64_t)tot[i];
    s = wave_sum_i64(s);
    const int nw = (blockDim.x + 63) >> 6;
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = s;
    __syncthreads();
    int64_t all = 0;
    for (int w = 0; w < nw; ++w) all += sh[w];
    __syncthreads();
    return all;
}

// What lies before chunk (or block) `c` of a sequence whose chunk totals are in tot[]: their sum, or, when the
// totals were already turned into prefixes by a scan of their own (more than `fused_max` of them), tot[c].
template <typename T>
__device__ inline int64_t prefix_before(const T* __restrict__ tot, int64_t c, int scanned, int64_t* sh) {
    if (scanned) return (int64_t)tot[c];
    return block_sum_of(tot, c, sh);
}

// ---- prefix sums in one block (the arrays here have 10^3 .. 10^6 entries) ---------------------
template <typename T> struct PtrLoad {
    const T* p;
    __device__ T operator()(int64_t i) const { return p[i]; }
};

template <typename Load, typename Out>
__global__ __launch_bounds__(1024) void k_scan_block(Load in, Out* __restrict__ out, int64_t n) {
    __shared__ int64_t wave_tot[16];
    constexpr int ITEMS = 4;
    Out carry = 0;
    for (int64_t base = 0; base < n; base += 1024 * ITEMS) {
        const int64_t i0 = base + (int64_t)threadIdx.x * ITEMS;
        Out v[ITEMS];
        int64_t sum = 0;
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) {
            v[j] = i0 + j < n ? (Out)in(i0 + j) : (Out)0;
            sum += (int64_t)v[j];
        }
        int64_t total;
        Out run = carry + (Out)block_excl_scan(sum, &total, wave_tot);
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) {
            if (i0 + j < n) out[i0 + j] = run;
            run += v[j];
        }
        carry += (Out)total;
    }
}

// ---- a0: counts ----------------------------------------------------------------------------
// Per-query counters live in LDS while a block walks its share of the request and are flushed
// once; the per-node counters and the touched-node bitmap take the global atomics directly
// (their addresses are spread over the whole graph).
template <bool LDS_Q, int EDGE_ITEMS, bool BIT_FIRST>
__global__ __launch_bounds__(EDGE_BLOCK) void k_count(const int32_t* __restrict__ qe_query,
                                                     const int32_t* __restrict__ qe_node, int64_t n_e,
                                                     int32_t n_query, int64_t n_nodes, int32_t* __restrict__ qcnt,
                                                     omg_ctx::NodeRec* __restrict__ node, uint32_t* __restrict__ bitmap,
                                                     uint32_t* __restrict__ bitmap1, BuildCounts* c) {
    extern __shared__ int32_t lq[];
    if (LDS_Q) {
        for (int i = threadIdx.x; i < n_query; i += (int)blockDim.x) lq[i] = 0;
        __syncthreads();
    }
    const int64_t e0 = (int64_t)blockIdx.x * (int)blockDim.x * EDGE_ITEMS;
    bool bad = false;
#pragma unroll
    for (int k = 0; k < EDGE_ITEMS; ++k) {
        const int64_t i = e0 + (int64_t)k * (int)blockDim.x + threadIdx.x;
        if (i >= n_e) break;
        const int32_t q = qe_query[i], u = qe_node[i];
        if (q < 0 || q >= n_query || u < 0 || (int64_t)u >= n_nodes) {
            bad = true;                      // the build is rejected after the read-back; this edge is left out
            continue;
        }
        if (LDS_Q) atomicAdd(&lq[q], 1);
        else atomicAdd(&qcnt[q], 1);
        if constexpr (BIT_FIRST) {
            // The node's bit tells the first edge at a node from the later ones: exactly one edge finds it unset.
            // Only the later ones touch the node's record (cnt = request edges at the node beyond the first).  For
            // requests that reach few of the graph's nodes: most candidates then have one request edge, the bitmap
            // is a thirty-second of the records' size and stays in the caches, and an atomic on a record of a large
            // graph is a trip to HBM (111 M nodes, 0.49 M edges: graph construction -15 us).
            const uint32_t bit = 1u << (u & 31);
            const uint32_t before = atomicOr(&bitmap[u >> 5], bit);
            if (before & bit) {
                atomicAdd(&node[u].cnt, 1);
            } else if (bitmap1 != nullptr && before == 0u) {
                // second level (large graphs only): one bit per word of the node bitmap, set by whoever finds the word empty
                atomicOr(&bitmap1[u >> 10], 1u << ((u >> 5) & 31));
            }
        } else {
            // Every edge counts at its node; the one that finds the counter at zero sets the node's bit.  For requests
            // with many edges per node of the graph: the records stay in L2, and the bitmap's few words would be hit
            // by dozens of returning atomics each (230 k nodes, 0.48 M edges: +8 us with the form above).
            if (atomicAdd(&node[u].cnt, 1) == 0) {
                const uint32_t before = atomicOr(&bitmap[u >> 5], 1u << (u & 31));
                if (bitmap1 != nullptr && before == 0u) atomicOr(&bitmap1[u >> 10], 1u << ((u >> 5) & 31));
            }
        }
    }
    if (bad) atomicOr(&c->err, 1);
    if (LDS_Q) {
        __syncthreads();
        for (int i = threadIdx.x; i < n_query; i += (int)blockDim.x)
            if (lq[i]) atomicAdd(&qcnt[i], lq[i]);
    }
}

// ---- a1: ranking key -----------------------------------------------------------------------
// floor(2^64 a / (a + b)) for 1 <= a, a + b < 2^32: two different ratios with denominators below
// 2^32 differ by more than 2^-64, so this 64-bit key orders them exactly; b == 0 (ratio 1) maps
// to the all-ones key, above every other value.  With denominators below 2^m the top 2m bits
// are already enough.
__device__ inline uint64_t ratio_key(uint64_t a, uint64_t b) {
    if (b == 0) return ~0ull;
    const uint64_t d = a + b;
    const uint64_t hi = (a << 32) / d;
    const uint64_t rem = (a << 32) - hi * d;
    const uint64_t lo = (rem << 32) / d;
    return (hi << 32) | lo;
}

// Keys of the alternative policies (Sec. 5.2.2), larger = recomputed first, in the top bits of 64:
// RANDOM: the top 39 bits of the splitmix64 finaliser of seed * C + node id (a counter-based generator, so
// that any implementation draws the same numbers); SCORE: a per-node fp32 score mapped to an unsigned
// integer of the same order (-0 counts as +0).
__device__ inline uint64_t random_key(uint64_t seed, uint32_t u) {
    uint64_t z = (uint64_t)u + seed * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    z = z ^ (z >> 31);
    return z & ~((1ull << 25) - 1ull);
}
__device__ inline uint64_t score_key(float x) {
    uint32_t b = x == 0.f ? 0u : __float_as_uint(x);
    b = (b & 0x80000000u) ? ~b : (b | 0x80000000u);
    return (uint64_t)b << 32;
}

// popcount totals of every chunk of 64 words of a bitmap (a wavefront per chunk)
__global__ __launch_bounds__(1024) void k_popc_chunks(const uint32_t* __restrict__ w, int64_t n_words,
                                                      int32_t* __restrict__ chunk_tot) {
    const int64_t i = gtid();
    int64_t c = i < n_words ? __popc(w[i]) : 0;
    c = wave_sum_i64(c);
    if ((threadIdx.x & 63) == 0 && (i >> 6) <= ((n_words - 1) >> 6)) chunk_tot[i >> 6] = (int32_t)c;
}

// Large graphs: the words of the node bitmap that hold a candidate, in ascending order, from the second-level
// bitmap (one thread per second-level word), with each word's popcount.  Walking n / 32 words per batch costs
// more than the whole rest of a small batch once n is 10^8; this way only n / 1024 words are walked.  Clears the
// second level.  Where a listed word goes: the set bits before this second-level word, from the chunk totals of
// k_popc_chunks (a wavefront is a chunk).
__global__ __launch_bounds__(TPB) void k_list_words(uint32_t* __restrict__ bitmap1,
                                                    const int32_t* __restrict__ chunk_tot, int chunk_scanned, int64_t n_words1,
                                                    const uint32_t* __restrict__ bitmap, int32_t* __restrict__ word_list,
                                                    int32_t* __restrict__ word_cnt, DevState* st) {
    const int64_t i = gtid();                             // no early return: wavefront-wide sums below
    const int lane = threadIdx.x & 63;
    uint32_t m = i < n_words1 ? bitmap1[i] : 0u;
    const int pc = __popc(m);
    int incl = pc;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int y = __shfl_up(incl, d);
        if (lane >= d) incl += y;
    }
    const int64_t chunk = i >> 6;                         // the same in every lane of the wavefront
    const int64_t last_chunk = (n_words1 - 1) >> 6;
    int64_t before = 0;
    if (chunk_scanned) {
        before = chunk_tot[chunk <= last_chunk ? chunk : 0];
    } else {
        for (int64_t j = lane; j < chunk && j <= last_chunk; j += 64) before += chunk_tot[j];
        before = wave_sum_i64(before);
    }
    int64_t at = before + incl - pc;
    if (i == n_words1 - 1) st->n_touched_words = at + pc;
    if (m == 0u) return;
    bitmap1[i] = 0u;
    while (m) {
        const int b = __ffs((int)m) - 1;
        m &= m - 1u;
        const int32_t w = (int32_t)(i * 32 + b);
        word_list[at] = w;
        word_cnt[at] = __popc(bitmap[w]);
        ++at;
    }
}

// totals of every chunk of 64 listed words' popcounts (zero past the end of the list)
__global__ __launch_bounds__(1024) void k_list_chunks(const int32_t* __restrict__ word_cnt, const DevState* st,
                                                      int64_t max_touched, int32_t* __restrict__ chunk_tot) {
    const int64_t i = gtid();
    const int64_t n = st->n_touched_words;
    int64_t c = i < n ? word_cnt[i] : 0;
    c = wave_sum_i64(c);
    if ((threadIdx.x & 63) == 0 && i < max_touched + 64) chunk_tot[i >> 6] = (int32_t)c;
}

// bitmap -> candidates in ascending id, one thread per byte of a bitmap word (a block covers 64 words); also returns
// the bitmap to its idle state.  The set bits a wavefront finds are first listed in LDS and then handled one per lane:
// where few bits are set, walking the eight bits of a byte in every lane would run the per-candidate work (three
// dependent loads and a 64-bit division) eight times with a handful of lanes active.  The words are all n_words of
// the bitmap (word_list == nullptr), or the listed ones.  A candidate's place in R = the set bits before it: those of
// the earlier blocks from the chunk totals (k_popc_chunks / k_list_chunks); the block's own 64 words are scanned here.
__global__ __launch_bounds__(TPB) void k_emit_candidates(uint32_t* __restrict__ bitmap,
                                  const int32_t* __restrict__ chunk_tot, int chunk_scanned,
                                  int64_t n_words, const int32_t* __restrict__ word_list, const DevState* st,
                                  omg_ctx::NodeRec* __restrict__ node, int32_t* __restrict__ cand,
                                  int32_t* __restrict__ qdeg, uint64_t* __restrict__ skey, BuildCounts* c, int policy,
                                  uint64_t seed, const float* __restrict__ node_scores, int bit_first) {
    // (node, place in R) of the set bits a wavefront found, so that the per-candidate work below runs on full
    // wavefronts also where the bitmap is sparse (a wavefront covers 512 node ids)
    __shared__ int32_t s_node[TPB / 64][512];
    __shared__ int32_t s_rank[TPB / 64][512];
    __shared__ int64_t s_red[16];
    __shared__ int32_t s_wpre[65];
    const int64_t t = gtid();
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int64_t e = t >> 2;                         // entry of the prefix sums
    const int64_t e0 = (int64_t)blockIdx.x * (TPB / 4);
    if (word_list != nullptr) n_words = st->n_touched_words;
    if (e0 >= n_words) {                              // the whole block lies past the last word
        if (t == 0) c->n_cand = 0;
        return;
    }
    const int64_t base = prefix_before(chunk_tot, (int64_t)blockIdx.x, chunk_scanned, s_red);
    {
        if (threadIdx.x < 64) {                       // the block's own 64 words
            const int64_t ee = e0 + threadIdx.x;
            const int pc = ee < n_words ? __popc(bitmap[word_list != nullptr ? word_list[ee] : ee]) : 0;
            int incl = pc;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const int y = __shfl_up(incl, d);
                if (lane >= d) incl += y;
            }
            s_wpre[threadIdx.x] = incl - pc;
            if (threadIdx.x == 63) s_wpre[64] = incl;
        }
        __syncthreads();                              // the words are cleared only below, after these reads
        if (threadIdx.x == 0 && e0 + TPB / 4 >= n_words) c->n_cand = base + s_wpre[64];
    }
    uint32_t bits = 0u;
    int32_t r0 = 0;
    int64_t w = 0;
    const int sh = (int)(t & 3) * 8;
    if (e < n_words) {
        w = word_list != nullptr ? word_list[e] : e;
        const uint32_t word = bitmap[w];
        // The four threads of a word sit in one wavefront and have all read it by the time any of them gets
        // past this test (the branch needs the loaded value), so the first of them may clear it.
        if (word != 0 && (t & 3) == 0) bitmap[w] = 0;
        bits = (word >> sh) & 0xffu;
        if (bits != 0u)
            r0 = (int32_t)base + s_wpre[e - e0] + __popc(word & ((1u << sh) - 1u));
    }
    const int mine = __popc(bits);
    int incl = mine;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int y = __shfl_up(incl, d);
        if (lane >= d) incl += y;
    }
    const int total = __shfl(incl, 63);
    int at = incl - mine;
    while (bits) {
        const int b = __ffs((int)bits) - 1;
        bits &= bits - 1u;
        s_node[wv][at] = (int32_t)(w * 32 + sh + b);
        s_rank[wv][at] = r0++;
        ++at;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    for (int i = lane; i < total; i += 64) {
        const int32_t u = s_node[wv][i];
        const int32_t r = s_rank[wv][i];
        const int4 rec = *reinterpret_cast<const int4*>(&node[u]);       // slot, cnt, deg: one load
        const int32_t a = rec.y + bit_first;                             // (the first request edge may only have set the node's bit)
        *reinterpret_cast<int2*>(&node[u]) = make_int2(r, 0);          // slot = r, cnt back to 0: one store
        cand[r] = u;
        qdeg[r] = a;
        skey[r] = policy == OMG_POLICY_RANDOM ? random_key(seed, (uint32_t)u)
                  : policy == OMG_POLICY_SCORE ? score_key(node_scores[u])
                                               : ratio_key((uint64_t)a, (uint64_t)rec.z);
    }
}

// Radix select of the k-th largest key, most significant digit first.  Per digit two kernels:
// k_select_hist builds the histogram of the digit over the candidates that match the digits
// chosen so far (LDS per block, flushed to global bins); k_select_find (one block) walks
// the bins from the top down to the one that holds the k-th largest and clears them.
__global__ __launch_bounds__(1024) void k_select_hist(const uint64_t* __restrict__ skey, DevState* st, int pass) {
    __shared__ unsigned int lh[SEL_BINS];
    const int tid = threadIdx.x;
    const int hi = 64 - SEL_BITS * pass;
    const int lo = hi - SEL_BITS > 0 ? hi - SEL_BITS : 0;
    const uint64_t dmask = (1ull << (hi - lo)) - 1;
    const int64_t n = st->counts.n_cand;
    const uint64_t prefix = st->sel.prefix;
    const int64_t r0 = (int64_t)blockIdx.x * 1024 * SEL_ITEMS + tid;
    if ((int64_t)blockIdx.x * 1024 * SEL_ITEMS >= n) return;
    uint64_t key[SEL_ITEMS];
#pragma unroll
    for (int k = 0; k < SEL_ITEMS; ++k) key[k] = r0 + k * 1024 < n ? skey[r0 + k * 1024] : 0;
    for (int i = tid; i < SEL_BINS; i += 1024) lh[i] = 0;
    __syncthreads();
#pragma unroll
    for (int k = 0; k < SEL_ITEMS; ++k)
        if (r0 + k * 1024 < n && (pass == 0 || (key[k] >> hi) == prefix)) atomicAdd(&lh[(key[k] >> lo) & dmask], 1u);
    __syncthreads();
    for (int i = tid; i < SEL_BINS; i += 1024)
        if (lh[i]) atomicAdd(&st->hist[i], lh[i]);
}

__global__ __launch_bounds__(1024) void k_select_find(DevState* st, int pass, uint32_t gamma_ppm) {
    __shared__ int64_t wave_tot[16];
    const int tid = threadIdx.x;
    const int hi = 64 - SEL_BITS * pass;
    const int lo = hi - SEL_BITS > 0 ? hi - SEL_BITS : 0;
    const int nb = hi - lo;
    constexpr int PER = SEL_BINS / 1024;
    const int top = SEL_BINS - PER * tid;         // this thread owns bins [top - PER, top), walked downwards
    unsigned int mine[PER];
    int64_t gsum = 0;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        mine[j] = st->hist[top - 1 - j];
        gsum += mine[j];
    }
#pragma unroll
    for (int j = 0; j < PER; ++j)
        if (mine[j]) st->hist[top - 1 - j] = 0u;
    const int64_t n = st->counts.n_cand;
    const uint64_t prefix = st->sel.prefix;
    long long k_rem = st->sel.k_rem;
    if (pass == 0) k_rem = (long long)(((uint64_t)gamma_ppm * (uint64_t)n) / 1000000ull);
    int64_t total;
    const int64_t before = block_excl_scan(gsum, &total, wave_tot);
    if (tid == 0 && pass == 0) {
        st->sel.k_take = k_rem;
        st->sel.take_none = k_rem == 0 ? 1 : 0;
        st->sel.n_list = 0;
        if (k_rem == 0) st->sel.k_rem = 0;
    }
    if (k_rem >= 1 && before < k_rem && k_rem <= before + gsum) {
        int64_t acc = before;
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            if (acc + mine[j] >= k_rem) {
                st->sel.prefix = (pass == 0 ? 0ull : (prefix << nb)) | (uint64_t)(top - 1 - j);
                st->sel.k_rem = k_rem - acc;
                break;
            }
            acc += mine[j];
        }
    }
}

// After the first digit few keys are left in the running (those of one bin out of 8,192; with the ratio policy most
// of them are ties: nodes with the same two degrees).  Instead of two more launches per further digit, all blocks
// copy the keys that match the first digit to a list (k_select_compact) and one block finishes the select on the
// list (k_select_rest): all keys equal -> done at once; else the remaining digits, the list's keys held in
// registers (the first 8,192 of them; a longer list is read again in every pass).
__global__ __launch_bounds__(1024) void k_select_compact(const uint64_t* __restrict__ skey, DevState* st,
                                                         uint64_t* __restrict__ list) {
    __shared__ int s_cnt[16];
    __shared__ long long s_base;
    if (st->sel.take_none) return;
    const int tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
    const int hi = 64 - SEL_BITS;
    const int64_t n = st->counts.n_cand;
    const uint64_t prefix = st->sel.prefix;
    const int64_t r0 = (int64_t)blockIdx.x * 1024 * SEL_ITEMS + tid;
    if ((int64_t)blockIdx.x * 1024 * SEL_ITEMS >= n) return;
    uint64_t key[SEL_ITEMS];
    bool match[SEL_ITEMS];
    int mine = 0;
#pragma unroll
    for (int k = 0; k < SEL_ITEMS; ++k) {
        key[k] = r0 + k * 1024 < n ? skey[r0 + k * 1024] : 0;
        match[k] = r0 + k * 1024 < n && (key[k] >> hi) == prefix;
        mine += match[k] ? 1 : 0;
    }
    int incl = mine;                                      // places inside the block: lanes, then wavefronts
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int y = __shfl_up(incl, d);
        if (lane >= d) incl += y;
    }
    if (lane == 63) s_cnt[wid] = incl;
    __syncthreads();
    if (tid == 0) {
        int tot = 0;
        for (int w = 0; w < 16; ++w) {
            const int c = s_cnt[w];
            s_cnt[w] = tot;
            tot += c;
        }
        s_base = tot ? (long long)atomicAdd((unsigned long long*)&st->sel.n_list, (unsigned long long)tot) : 0;
    }
    __syncthreads();
    int64_t at = s_base + s_cnt[wid] + incl - mine;
#pragma unroll
    for (int k = 0; k < SEL_ITEMS; ++k)
        if (match[k]) list[at++] = key[k];
}

__global__ __launch_bounds__(1024) void k_select_rest(const uint64_t* __restrict__ list, DevState* st, int n_pass,
                                                      int lo_final) {
    __shared__ unsigned int lh[SEL_BINS];
    __shared__ int64_t wave_tot[16];
    __shared__ unsigned long long s_red[2][16];
    __shared__ unsigned long long s_prefix;
    __shared__ long long s_krem;
    if (st->sel.take_none) return;
    constexpr int KPT = 8;
    const int tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
    const int64_t n = st->sel.n_list;
    uint64_t mk[KPT];
    uint64_t lo_key = ~0ull, hi_key = 0ull;
#pragma unroll
    for (int k = 0; k < KPT; ++k) {
        mk[k] = tid + k * 1024 < n ? list[tid + k * 1024] : 0;
        if (tid + k * 1024 < n) {
            lo_key = mk[k] < lo_key ? mk[k] : lo_key;
            hi_key = mk[k] > hi_key ? mk[k] : hi_key;
        }
    }
    for (int64_t i = (int64_t)KPT * 1024 + tid; i < n; i += 1024) {
        const uint64_t key = list[i];
        lo_key = key < lo_key ? key : lo_key;
        hi_key = key > hi_key ? key : hi_key;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const uint64_t a = __shfl_xor(lo_key, off), b = __shfl_xor(hi_key, off);
        lo_key = a < lo_key ? a : lo_key;
        hi_key = b > hi_key ? b : hi_key;
    }
    if (lane == 0) {
        s_red[0][wid] = lo_key;
        s_red[1][wid] = hi_key;
    }
    __syncthreads();
    for (int w = 0; w < 16; ++w) {
        lo_key = s_red[0][w] < lo_key ? s_red[0][w] : lo_key;
        hi_key = s_red[1][w] > hi_key ? s_red[1][w] : hi_key;
    }
    if (lo_key == hi_key) {                               // every key left is the same: all further digits are its digits
        if (tid == 0) st->sel.prefix = lo_key >> lo_final;
        return;
    }
    constexpr int PER = SEL_BINS / 1024;
    unsigned long long prefix = st->sel.prefix;
    long long k_rem = st->sel.k_rem;
    for (int pass = 1; pass < n_pass; ++pass) {
        const int hi = 64 - SEL_BITS * pass;
        const int lo = hi - SEL_BITS > 0 ? hi - SEL_BITS : 0;
        const int nb = hi - lo;
        const uint64_t dmask = (1ull << nb) - 1;
        for (int i = tid; i < SEL_BINS; i += 1024) lh[i] = 0;
        __syncthreads();
#pragma unroll
        for (int k = 0; k < KPT; ++k)
            if (tid + k * 1024 < n && (mk[k] >> hi) == prefix) atomicAdd(&lh[(mk[k] >> lo) & dmask], 1u);
        for (int64_t i = (int64_t)KPT * 1024 + tid; i < n; i += 1024) {
            const uint64_t key = list[i];
            if ((key >> hi) == prefix) atomicAdd(&lh[(key >> lo) & dmask], 1u);
        }
        __syncthreads();
        const int top = SEL_BINS - PER * tid;     // this thread owns bins [top - PER, top), walked downwards
        unsigned int mine[PER];
        int64_t gsum = 0;
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            mine[j] = lh[top - 1 - j];
            gsum += mine[j];
        }
        int64_t total;
        const int64_t before = block_excl_scan(gsum, &total, wave_tot);
        if (before < k_rem && k_rem <= before + gsum) {
            int64_t acc = before;
#pragma unroll
            for (int j = 0; j < PER; ++j) {
                if (acc + mine[j] >= k_rem) {
                    s_prefix = (prefix << nb) | (unsigned long long)(top - 1 - j);
                    s_krem = k_rem - acc;
                    break;
                }
                acc += mine[j];
            }
        }
        __syncthreads();
        prefix = s_prefix;
        k_rem = s_krem;
        __syncthreads();
    }
    if (tid == 0) {
        st->sel.prefix = prefix;
        st->sel.k_rem = k_rem;
    }
}

// The whole select in one block, for batches with few candidates: the same passes as above with the histogram in
// LDS only.  KPT > 0: every thread keeps its KPT keys (candidates tid, tid + 1024, ...) in registers over all passes
// (up to 32 K candidates); KPT == 0: every pass reads the keys again (up to SELECT_ONE_BLOCK_MAX of them; a pass is
// then a chain of dependent trips to memory: 25.7 us for 30 K candidates and four passes, 13 us from registers).
template <int KPT>
__global__ __launch_bounds__(1024) void k_select_all(const uint64_t* __restrict__ skey, DevState* st, int n_pass,
                                                     uint32_t gamma_ppm) {
    __shared__ unsigned int lh[SEL_BINS];
    __shared__ int64_t wave_tot[16];
    __shared__ unsigned long long s_prefix;
    __shared__ long long s_krem;
    const int tid = threadIdx.x;
    const int64_t n = st->counts.n_cand;
    const long long k_take = (long long)(((uint64_t)gamma_ppm * (uint64_t)n) / 1000000ull);
    if (tid == 0) {
        st->sel.k_take = k_take;
        st->sel.take_none = k_take == 0 ? 1 : 0;
        if (k_take == 0) st->sel.k_rem = 0;
    }
    if (k_take == 0) return;
    uint64_t mine_key[KPT > 0 ? KPT : 1];
    if constexpr (KPT > 0) {
#pragma unroll
        for (int k = 0; k < KPT; ++k) mine_key[k] = tid + k * 1024 < n ? skey[tid + k * 1024] : 0;
    }
    constexpr int PER = SEL_BINS / 1024;
    unsigned long long prefix = 0;
    long long k_rem = k_take;
    for (int pass = 0; pass < n_pass; ++pass) {
        const int hi = 64 - SEL_BITS * pass;
        const int lo = hi - SEL_BITS > 0 ? hi - SEL_BITS : 0;
        const int nb = hi - lo;
        const uint64_t dmask = (1ull << nb) - 1;
        for (int i = tid; i < SEL_BINS; i += 1024) lh[i] = 0;
        __syncthreads();
        if constexpr (KPT > 0) {
#pragma unroll
            for (int k = 0; k < KPT; ++k) {
                const uint64_t key = mine_key[k];
                if (tid + k * 1024 < n && (pass == 0 || (key >> hi) == prefix)) atomicAdd(&lh[(key >> lo) & dmask], 1u);
            }
        } else {
            for (int64_t i = tid; i < n; i += 1024) {
                const uint64_t key = skey[i];
                if (pass == 0 || (key >> hi) == prefix) atomicAdd(&lh[(key >> lo) & dmask], 1u);
            }
        }
        __syncthreads();
        const int top = SEL_BINS - PER * tid;     // this thread owns bins [top - PER, top), walked downwards
        unsigned int mine[PER];
        int64_t gsum = 0;
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            mine[j] = lh[top - 1 - j];
            gsum += mine[j];
        }
        int64_t total;
        const int64_t before = block_excl_scan(gsum, &total, wave_tot);
        if (before < k_rem && k_rem <= before + gsum) {
            int64_t acc = before;
#pragma unroll
            for (int j = 0; j < PER; ++j) {
                if (acc + mine[j] >= k_rem) {
                    s_prefix = (pass == 0 ? 0ull : (prefix << nb)) | (unsigned long long)(top - 1 - j);
                    s_krem = k_rem - acc;
                    break;
                }
                acc += mine[j];
            }
        }
        __syncthreads();
        prefix = s_prefix;
        k_rem = s_krem;
        __syncthreads();
    }
    if (tid == 0) {
        st->sel.prefix = prefix;
        st->sel.k_rem = k_rem;
    }
}

// per candidate: (key > threshold, key == threshold) packed for one prefix sum.  Thread 0 also resets the
// counters that later kernels accumulate into.
__device__ inline void reset_accumulators(BuildCounts* c) {
    c->n_target = 0;
    c->nnz_in = 0;
    c->n_parts = 0;
    c->n_parts_last = 0;
    c->n_split = 0;
    c->n_split_last = 0;
    c->n_split_big = 0;
    c->n_split_big_last = 0;
    c->n_small = 0;
    c->n_med = 0;
    c->n_big = 0;
}

// Blocks of SUM_BLOCK candidates; besides the flags, every block leaves its total (same packing) for k_targets.
__global__ __launch_bounds__(SUM_BLOCK) void k_flag(const uint64_t* __restrict__ skey, DevState* st, int lo_final,
                                                    int force_none, int64_t n_slots, uint64_t* __restrict__ flag,
                                                    uint64_t* __restrict__ flag_tot) {
    __shared__ int64_t sh[16];
    const int64_t r = gtid();
    if (r == 0) {
        reset_accumulators(&st->counts);
        for (int f = 0; f < ORDER_PHASES; ++f) st->phase_total[f * 8] = st->phase_rank[f * 8] = 0;
        if (force_none) {
            st->sel.take_none = 1;
            st->sel.k_rem = 0;
        }
    }
    uint64_t f = 0;
    if (r < n_slots && r < st->counts.n_cand && !force_none && !st->sel.take_none) {
        const uint64_t kk = skey[r] >> lo_final, thr = st->sel.prefix;
        f = kk > thr ? 1ull : (kk == thr ? (1ull << 32) : 0ull);
    }
    if (r < n_slots) flag[r] = f;
    const int64_t s = wave_sum_i64((int64_t)f);
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        int64_t all = 0;
        for (int w = 0; w < SUM_BLOCK / 64; ++w) all += sh[w];
        flag_tot[blockIdx.x] = (uint64_t)all;
    }
}

__global__ void k_zero_flags(DevState* st, int64_t n_slots, uint64_t* __restrict__ flag) {
    const int64_t r = gtid();
    if (r == 0) {
        reset_accumulators(&st->counts);
        for (int f = 0; f < ORDER_PHASES; ++f) st->phase_total[f * 8] = st->phase_rank[f * 8] = 0;
        st->sel.take_none = 0;
        st->sel.k_rem = 0;          // an explicit set has no "first few of the equal ones"
    }
    if (r < n_slots) flag[r] = 0;
}

__global__ void k_mark_given(const int32_t* __restrict__ rset, int64_t n_rset, int64_t n_nodes,
                             const omg_ctx::NodeRec* __restrict__ node, uint64_t* __restrict__ flag, BuildCounts* c) {
    const int64_t t = gtid();
    if (t >= n_rset) return;
    const int32_t u = rset[t];
    const bool ok = u >= 0 && (int64_t)u < n_nodes && (t == 0 || rset[t - 1] < u);
    const int32_t r = ok ? node[u].slot : -1;
    if (r < 0) atomicOr(&c->err, 2);
    else flag[r] = 1ull;
}

// block totals of flags that were written one by one (an explicit recompute set)
__global__ __launch_bounds__(SUM_BLOCK) void k_flag_totals(const uint64_t* __restrict__ flag, int64_t n_slots,
                                                           uint64_t* __restrict__ flag_tot) {
    __shared__ int64_t sh[16];
    const int64_t r = gtid();
    const int64_t s = wave_sum_i64(r < n_slots ? (int64_t)flag[r] : 0);
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        int64_t all = 0;
        for (int w = 0; w < SUM_BLOCK / 64; ++w) all += sh[w];
        flag_tot[blockIdx.x] = (uint64_t)all;
    }
}

// targets in ascending id: all candidates above the threshold plus the first k_rem at it.  The flags before a
// candidate = the totals of the earlier blocks (k_flag's blocks) + a scan inside the block.
__global__ __launch_bounds__(SUM_BLOCK) void k_targets(const int32_t* __restrict__ cand, const int32_t* __restrict__ qdeg,
                          const uint64_t* __restrict__ flag, const uint64_t* __restrict__ flag_tot, int tot_scanned,
                          DevState* st, int32_t n_query, const int64_t* __restrict__ base_indptr,
                          int32_t* __restrict__ targets, int32_t* __restrict__ target_slot,
                          int32_t* __restrict__ cand_row, int32_t* __restrict__ tcur, int64_t* __restrict__ tlen) {
    __shared__ int64_t sh[16];
    const int64_t r = gtid();
    const int64_t n = st->counts.n_cand;
    if ((int64_t)blockIdx.x * SUM_BLOCK >= n) return;         // the whole block lies past the last candidate
    const uint64_t f = r < n ? flag[r] : 0ull;
    const int64_t before_blocks = prefix_before(flag_tot, (int64_t)blockIdx.x, tot_scanned, sh);
    int64_t total;
    const uint64_t s = (uint64_t)(before_blocks + block_excl_scan((int64_t)f, &total, sh));
    if (r >= n) return;
    const int64_t m = st->sel.k_rem;
    const int64_t gt_before = (int64_t)(s & 0xffffffffull), eq_before = (int64_t)(s >> 32);
    const bool gt = (f & 1ull) != 0, eq = (f >> 32) != 0;
    const bool in_t = gt || (eq && eq_before < m);
    const int64_t t = gt_before + (eq_before < m ? eq_before : m);
    if (in_t) {
        const int32_t u = cand[r];
        targets[t] = u;
        target_slot[t] = (int32_t)r;
        cand_row[r] = n_query + (int32_t)t;
        tcur[t] = 0;
        tlen[t] = base_deg(base_indptr, u) + qdeg[r];
    } else {
        cand_row[r] = -1;
    }
    if (r == n - 1) st->counts.n_target = t + (in_t ? 1 : 0);
}

// ---- a2: row lengths, work list sizes, sort work lists --------------------------------------

// Per row: its length and its number of parts (their prefix sums are the row pointers and the work list offsets:
// every block of SUM_BLOCK rows leaves its two totals for k_rowptr), its sorting class, and the batch totals.  Query
// rows come first; their lengths are the per-query counters, which are returned to zero here.  n_rows_b: an upper
// bound of the number of rows, plus one (the entry after the last row takes the end pointers).
__global__ __launch_bounds__(SUM_BLOCK) void k_rowlen(int32_t* __restrict__ qcnt, int32_t* __restrict__ qcur, const int64_t* __restrict__ tlen,
                         const int32_t* __restrict__ qdeg, const int32_t* __restrict__ target_slot, int32_t n_query,
                         int64_t n_rows_b, int part_edges, BuildCounts* c, int64_t* __restrict__ rowlen,
                         int32_t* __restrict__ nparts, int64_t* __restrict__ tot_len, int64_t* __restrict__ tot_np,
                         int32_t* __restrict__ list_small,
                         int32_t* __restrict__ list_med, int32_t* __restrict__ list_big,
                         int32_t* __restrict__ split_rows, int32_t* __restrict__ split_rows_q,
                         int32_t* __restrict__ split_big, int32_t* __restrict__ split_big_q,
                         long long* __restrict__ phase_total) {
    // Everything this kernel counts goes through LDS first: a block adds to each of the batch's counters once (the
    // three sizes, the eight region totals, the seven list cursors).  One atomic per wavefront and counter - 18 hot
    // addresses hit by every wavefront of the launch - was most of this kernel's time.
    constexpr int NW = SUM_BLOCK / 64;
    __shared__ int64_t sh_len[NW], sh_np[NW], sh_npq[NW];
    __shared__ int64_t sh_phase[ORDER_PHASES][NW];
    __shared__ int sh_cnt[7][NW];                     // per list: rows of each wavefront, then where its rows start
    __shared__ long long sh_base[7];
    const int64_t v = gtid();                         // no early return: the wavefront helpers need every lane
    const int lane = threadIdx.x & 63, wid = threadIdx.x >> 6;
    const int64_t rows_in = n_query + c->n_target;
    int64_t len = 0, seg = 0;
    int32_t np = 0;
    if (v < n_query) {
        len = qcnt[v];
        qcnt[v] = 0;
        qcur[v] = 0;
        seg = len;
    } else if (v < rows_in) {
        len = tlen[v - n_query];
        seg = qdeg[target_slot[v - n_query]];
    }
    if (v < rows_in) {
        const int ps = omg_row_part(len, part_edges);
        np = (int32_t)((len + ps - 1) / ps);
        if (np < 1) np = 1;
    }
    if (v < n_rows_b) {
        rowlen[v] = len;
        nparts[v] = np;
    }
    const int64_t s_len = wave_sum_i64(len), s_np = wave_sum_i64(np), s_npq = wave_sum_i64(v < n_query ? np : 0);
    // work items per region of the table: the k-th of np parts belongs to the f with first(f) <= k < first(f + 1)
    int64_t s_f[ORDER_PHASES];
#pragma unroll
    for (int f = 0; f < ORDER_PHASES; ++f) s_f[f] = wave_sum_i64(phase_first(f + 1, np) - phase_first(f, np));
    // seven lists take the rows: the rows cut into few / many parts (all, and the query rows among them), and the
    // rows by the size of what has to be sorted in them
    const bool few = np > 1 && np <= OMG_MANY_PARTS, many = np > OMG_MANY_PARTS;
    const bool small = seg >= 1 && seg <= SORT_WAVE_MAX;
    const bool med = seg > SORT_WAVE_MAX && seg <= SORT_MED_MAX;
    const bool big = seg > SORT_MED_MAX;
    const bool is_q = v < n_query;
    const unsigned long long m0 = __ballot(few), m1 = __ballot(few && is_q), m2 = __ballot(many),
                             m3 = __ballot(many && is_q), m4 = __ballot(small), m5 = __ballot(med), m6 = __ballot(big);
    if (lane == 0) {
        sh_len[wid] = s_len;
        sh_np[wid] = s_np;
        sh_npq[wid] = s_npq;
#pragma unroll
        for (int f = 0; f < ORDER_PHASES; ++f) sh_phase[f][wid] = s_f[f];
        sh_cnt[0][wid] = __popcll(m0); sh_cnt[1][wid] = __popcll(m1); sh_cnt[2][wid] = __popcll(m2);
        sh_cnt[3][wid] = __popcll(m3); sh_cnt[4][wid] = __popcll(m4); sh_cnt[5][wid] = __popcll(m5);
        sh_cnt[6][wid] = __popcll(m6);
    }
    __syncthreads();
    const int t = threadIdx.x;
    if (t == 0) {
        int64_t a = 0, b = 0, q = 0;
        for (int w = 0; w < NW; ++w) {
            a += sh_len[w];
            b += sh_np[w];
            q += sh_npq[w];
        }
        tot_len[blockIdx.x] = a;
        tot_np[blockIdx.x] = b;
        if (a) atomicAdd((unsigned long long*)&c->nnz_in, (unsigned long long)a);
        if (b) atomicAdd((unsigned long long*)&c->n_parts, (unsigned long long)b);
        if (q) atomicAdd((unsigned long long*)&c->n_parts_last, (unsigned long long)q);
    } else if (t >= 64 && t < 64 + ORDER_PHASES) {
        const int f = t - 64;
        int64_t a = 0;
        for (int w = 0; w < NW; ++w) a += sh_phase[f][w];
        if (a) atomicAdd((unsigned long long*)&phase_total[f * 8], (unsigned long long)a);
    } else if (t >= 128 && t < 128 + 7) {
        const int j = t - 128;
        int tot = 0;
        for (int w = 0; w < NW; ++w) {
            const int n = sh_cnt[j][w];
            sh_cnt[j][w] = tot;
            tot += n;
        }
        long long* const ctr = j == 0 ? (long long*)&c->n_split : j == 1 ? (long long*)&c->n_split_last
                               : j == 2 ? (long long*)&c->n_split_big : j == 3 ? (long long*)&c->n_split_big_last
                               : j == 4 ? (long long*)&c->n_small : j == 5 ? (long long*)&c->n_med : (long long*)&c->n_big;
        sh_base[j] = tot ? (long long)atomicAdd((unsigned long long*)ctr, (unsigned long long)tot) : 0;
    }
    __syncthreads();
    const unsigned long long below = (1ull << lane) - 1ull;
    if (few) split_rows[sh_base[0] + sh_cnt[0][wid] + __popcll(m0 & below)] = (int32_t)v;
    if (few && is_q) split_rows_q[sh_base[1] + sh_cnt[1][wid] + __popcll(m1 & below)] = (int32_t)v;
    if (many) split_big[sh_base[2] + sh_cnt[2][wid] + __popcll(m2 & below)] = (int32_t)v;
    if (many && is_q) split_big_q[sh_base[3] + sh_cnt[3][wid] + __popcll(m3 & below)] = (int32_t)v;
    if (small) list_small[sh_base[4] + sh_cnt[4][wid] + __popcll(m4 & below)] = (int32_t)v;
    if (med) list_med[sh_base[5] + sh_cnt[5][wid] + __popcll(m5 & below)] = (int32_t)v;
    if (big) list_big[sh_base[6] + sh_cnt[6][wid] + __popcll(m6 & below)] = (int32_t)v;
}

// Row pointers and work list offsets: exclusive prefix sums of (row length, parts per row), from the block totals of
// k_rowlen and a scan inside the block.  The first thread also hands the batch's sizes to the host (mailbox: pinned
// host memory as the device sees it), which is waiting for the build's number to appear there.
__global__ __launch_bounds__(SUM_BLOCK) void k_rowptr(const int64_t* __restrict__ rowlen, const int32_t* __restrict__ nparts,
                                                      int64_t n_rows_b, const int64_t* __restrict__ tot_len,
                                                      const int64_t* __restrict__ tot_np, int tot_scanned,
                                                      int64_t* __restrict__ indptr, int32_t* __restrict__ part_ptr,
                                                      const BuildCounts* __restrict__ c, HostMailbox* __restrict__ mailbox,
                                                      unsigned long long seq, int n_row_blocks, InitBufferArgs init) {
    __shared__ int64_t sh[16];
    if ((int)blockIdx.x >= n_row_blocks) {
        // The blocks behind those of the prefix sums fill the layer-0 buffer, which needs the targets and nothing
        // else of this kernel: a launch of its own would run after this one instead of beside it.  128 threads a row.
        constexpr int PER = SUM_BLOCK / 128;
        omg_init_buffer_rows(init, (int64_t)((int)blockIdx.x - n_row_blocks) * PER + (threadIdx.x >> 7),
                             (int64_t)((int)gridDim.x - n_row_blocks) * PER, (int)(threadIdx.x & 127), 128);
        return;
    }
    const int64_t i = gtid();
    if (i == 0 && mailbox != nullptr) {               // the sizes are final once k_rowlen is done: no need to wait for this kernel
        mailbox->counts = *c;
        __threadfence_system();
        __hip_atomic_store(&mailbox->seq, seq, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
    }
    const int64_t a = i < n_rows_b ? rowlen[i] : 0, b = i < n_rows_b ? nparts[i] : 0;
    const int64_t pa = prefix_before(tot_len, (int64_t)blockIdx.x, tot_scanned, sh);
    const int64_t pb = prefix_before(tot_np, (int64_t)blockIdx.x, tot_scanned, sh);
    int64_t ta, tb;
    const int64_t ea = block_excl_scan(a, &ta, sh);
    const int64_t eb = block_excl_scan(b, &tb, sh);
    if (i < n_rows_b) {
        indptr[i] = pa + ea;
        part_ptr[i] = (int32_t)(pb + eb);
    }
}

// ---- a2: columns -----------------------------------------------------------------------------
// Every request edge goes into its query row (as a node id) and, if its node is a target, into the
// tail of that target's row (as a query index).  Slots inside a query row are handed out from LDS:
// a block counts its edges per query, reserves that many slots per query with one global atomic,
// then numbers its own edges.  The order inside a row is fixed afterwards by the sorts.
template <bool LDS_Q, int EDGE_ITEMS>
__global__ __launch_bounds__(EDGE_BLOCK) void k_bucket(const int32_t* __restrict__ qe_query,
                                                      const int32_t* __restrict__ qe_node, int64_t n_e,
                                                      const int64_t* __restrict__ indptr,
                                                      const omg_ctx::NodeRec* __restrict__ node,
                                                      const int32_t* __restrict__ cand_row,
                                                      int32_t* __restrict__ qcur, int32_t* __restrict__ tcur,
                                                      int32_t n_query, int32_t* __restrict__ raw) {
    extern __shared__ int32_t lq[];
    const int64_t e0 = (int64_t)blockIdx.x * (int)blockDim.x * EDGE_ITEMS;
    int32_t q[EDGE_ITEMS], u[EDGE_ITEMS];
#pragma unroll
    for (int k = 0; k < EDGE_ITEMS; ++k) {
        const int64_t i = e0 + (int64_t)k * (int)blockDim.x + threadIdx.x;
        q[k] = i < n_e ? qe_query[i] : -1;
        u[k] = i < n_e ? qe_node[i] : 0;
    }
    if (LDS_Q) {
        for (int i = threadIdx.x; i < n_query; i += (int)blockDim.x) lq[i] = 0;
        __syncthreads();
#pragma unroll
        for (int k = 0; k < EDGE_ITEMS; ++k)
            if (q[k] >= 0) atomicAdd(&lq[q[k]], 1);
        __syncthreads();
        for (int i = threadIdx.x; i < n_query; i += (int)blockDim.x)
            if (lq[i]) lq[i] = atomicAdd(&qcur[i], lq[i]);   // count -> first slot of this block in row i
        __syncthreads();
    }
#pragma unroll
    for (int k = 0; k < EDGE_ITEMS; ++k) {
        if (q[k] < 0) continue;
        const int32_t pos = LDS_Q ? atomicAdd(&lq[q[k]], 1) : atomicAdd(&qcur[q[k]], 1);
        raw[indptr[q[k]] + pos] = u[k];
        const int4 rec = *reinterpret_cast<const int4*>(&node[u[k]]);    // slot and degree: one load
        const int32_t row = cand_row[rec.x];
        if (row >= 0) raw[indptr[row] + rec.z + atomicAdd(&tcur[row - n_query], 1)] = q[k];
    }
}

__device__ inline void segment_of(int32_t v, int32_t n_query, const int64_t* __restrict__ indptr,
                                  const int32_t* __restrict__ qdeg, const int32_t* __restrict__ target_slot,
                                  int64_t* s, int64_t* e) {
    *e = indptr[v + 1];
    *s = v < n_query ? indptr[v] : *e - qdeg[target_slot[v - n_query]];
}

// segments of 1..64 keys: one wavefront each, bitonic network over the lanes.  `block`: which block of TPB / 64
// segments of the list (the kernels below give their own index or a share of a larger grid).
__device__ inline void segsort_wave_body(int64_t block, const int32_t* __restrict__ list, int64_t n_list, int32_t n_query,
                                         const int64_t* __restrict__ indptr, const int32_t* __restrict__ qdeg,
                                         const int32_t* __restrict__ target_slot,
                                         const int32_t* __restrict__ raw, int32_t* __restrict__ cols) {
    const int lane = threadIdx.x & 63;
    const int64_t w = block * (TPB / 64) + (threadIdx.x >> 6);
    if (w >= n_list) return;
    int64_t s, e;
    segment_of(list[w], n_query, indptr, qdeg, target_slot, &s, &e);
    const int len = (int)(e - s);
    int32_t x = lane < len ? raw[s + lane] : 0x7fffffff;
    if (len > 1) {
#pragma unroll
        for (int k = 2; k <= 64; k <<= 1)
#pragma unroll
            for (int j = k >> 1; j > 0; j >>= 1) {
                const int32_t y = __shfl_xor(x, j);
                const bool up = (lane & k) == 0;
                const bool lower = (lane & j) == 0;
                x = (lower == up) ? (x < y ? x : y) : (x > y ? x : y);
            }
    }
    if (lane < len) cols[s + lane] = x;
}

// Longer segments: one block each, least-significant-digit radix sort with 4-bit digits, ping-pong
// between the two buffers.  Each thread owns a contiguous chunk of the segment (so every pass is
// stable) and keeps up to SORT_KEYS of its keys in registers between the counting and the
// scattering loop; its 16 digit counters are a column of an LDS matrix, scanned digit-major.
//
// Segments of more than SORT_MED_MAX keys first go through one pass on their TOP four bits
// (SPLIT = true, 1024 threads), which cuts them into 16 independent pieces; the pieces are then
// sorted on the remaining bits by the same blocks that sort the medium segments.
struct SubSeg {
    int64_t start;      // absolute offset into the column arrays
    int32_t len;
    int32_t bits;       // key bits that still have to be sorted
};

template <int THREADS, bool SPLIT>
__device__ inline void segsort_radix_body(int64_t block, const int32_t* __restrict__ list, int64_t n_list,
                                          int32_t n_query, const int64_t* __restrict__ indptr,
                                          const int32_t* __restrict__ qdeg,
                                          const int32_t* __restrict__ target_slot, int bits_node,
                                          int bits_query, SubSeg* __restrict__ sub, int64_t n_sub,
                                          int32_t* __restrict__ raw, int32_t* __restrict__ cols) {
    __shared__ int32_t cnt[16 * THREADS];
    __shared__ int64_t wave_tot[16];
    int64_t s, e;
    int bits;
    int32_t* src = raw;
    int32_t* dst = cols;
    if (block < n_list) {
        const int32_t v = list[block];
        segment_of(v, n_query, indptr, qdeg, target_slot, &s, &e);
        bits = v < n_query ? bits_node : bits_query;
    } else {
        if (SPLIT || block - n_list >= n_sub) return;
        const SubSeg g = sub[block - n_list];        // a piece of a split segment: its keys are in `cols`
        s = g.start;
        e = g.start + g.len;
        bits = g.bits;
        src = cols;
        dst = raw;
        if (g.len <= 1) return;
    }
    const int64_t len = e - s;
    const int t = threadIdx.x;
    const int64_t per = (len + THREADS - 1) / THREADS;
    const int64_t c0 = s + (int64_t)t * per < e ? s + (int64_t)t * per : e;
    const int64_t c1 = c0 + per < e ? c0 + per : e;
    const bool in_regs = per <= SORT_KEYS;
    if constexpr (!SPLIT) {
        // Segments that fit LDS (all the medium ones, and the pieces of most split ones) stay there between the
        // passes: a pass then costs three barriers instead of a round trip through global memory.
        __shared__ int32_t keys_lds[THREADS * SORT_KEYS];
        if (len <= THREADS * SORT_KEYS && bits > 0) {
            int32_t k[SORT_KEYS];
#pragma unroll
            for (int i = 0; i < SORT_KEYS; ++i) k[i] = c0 + i < c1 ? src[c0 + i] : -1;
            for (int shift = 0; shift < bits; shift += 4) {
#pragma unroll
                for (int d = 0; d < 16; ++d) cnt[d * THREADS + t] = 0;
#pragma unroll
                for (int i = 0; i < SORT_KEYS; ++i)
                    if (k[i] >= 0) cnt[((k[i] >> shift) & 15) * THREADS + t] += 1;
                __syncthreads();
                int32_t mine[16];
                int64_t sum = 0;
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    mine[j] = cnt[16 * t + j];
                    sum += mine[j];
                }
                int64_t total;
                int64_t run = block_excl_scan(sum, &total, wave_tot);
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    cnt[16 * t + j] = (int32_t)run;
                    run += mine[j];
                }
                __syncthreads();
#pragma unroll
                for (int i = 0; i < SORT_KEYS; ++i)
                    if (k[i] >= 0) {
                        const int slot = ((k[i] >> shift) & 15) * THREADS + t;
                        keys_lds[cnt[slot]] = k[i];
                        cnt[slot] += 1;
                    }
                __syncthreads();
                // this thread's share of the new order; the next pass writes keys_lds only after two more barriers
#pragma unroll
                for (int i = 0; i < SORT_KEYS; ++i) k[i] = c0 + i < c1 ? keys_lds[c0 - s + i] : -1;
            }
            for (int64_t i = t; i < len; i += THREADS) cols[s + i] = keys_lds[i];
            return;
        }
    }
    const int first_shift = SPLIT ? (bits > 4 ? bits - 4 : 0) : 0;
    const int end_shift = SPLIT ? first_shift + 1 : bits;
    for (int shift = first_shift; shift < end_shift; shift += 4) {
#pragma unroll
        for (int d = 0; d < 16; ++d) cnt[d * THREADS + t] = 0;
        int32_t k[SORT_KEYS];
        for (int64_t b0 = c0; b0 < c1; b0 += SORT_KEYS) {
#pragma unroll
            for (int i = 0; i < SORT_KEYS; ++i) k[i] = b0 + i < c1 ? src[b0 + i] : -1;
#pragma unroll
            for (int i = 0; i < SORT_KEYS; ++i)
                if (k[i] >= 0) cnt[((k[i] >> shift) & 15) * THREADS + t] += 1;
        }
        __syncthreads();
        // exclusive prefix sum over the digit-major counter matrix: thread t owns entries [16 t, 16 t + 16)
        int32_t mine[16];
        int64_t sum = 0;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            mine[j] = cnt[16 * t + j];
            sum += mine[j];
        }
        int64_t total;
        int64_t run = block_excl_scan(sum, &total, wave_tot);
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            cnt[16 * t + j] = (int32_t)run;
            run += mine[j];
        }
        __syncthreads();
        if (SPLIT && t < 16) {                   // where the 16 pieces start: the first thread's offsets
            const int32_t a = cnt[t * THREADS];
            const int32_t b = t < 15 ? cnt[(t + 1) * THREADS] : (int32_t)len;
            sub[block * 16 + t] = SubSeg{s + a, b - a, first_shift};
        }
        if (SPLIT) __syncthreads();
        for (int64_t b0 = c0; b0 < c1; b0 += SORT_KEYS) {
            if (!in_regs) {
#pragma unroll
                for (int i = 0; i < SORT_KEYS; ++i) k[i] = b0 + i < c1 ? src[b0 + i] : -1;
            }
#pragma unroll
            for (int i = 0; i < SORT_KEYS; ++i)
                if (k[i] >= 0) {
                    const int slot = ((k[i] >> shift) & 15) * THREADS + t;
                    dst[s + cnt[slot]] = k[i];
                    cnt[slot] += 1;
                }
        }
        __threadfence_block();
        __syncthreads();
        int32_t* sw = src;
        src = dst;
        dst = sw;
    }
    if (!SPLIT && src != cols)
        for (int64_t i = c0; i < c1; ++i) cols[i] = src[i];
}

// the first pass of the longest segments (see above)
__global__ __launch_bounds__(1024) void k_segsort_split(const int32_t* __restrict__ list, int64_t n_list, int32_t n_query,
                                                        const int64_t* __restrict__ indptr, const int32_t* __restrict__ qdeg,
                                                        const int32_t* __restrict__ target_slot, int bits_node, int bits_query,
                                                        SubSeg* __restrict__ sub, int32_t* __restrict__ raw,
                                                        int32_t* __restrict__ cols) {
    segsort_radix_body<1024, true>((int64_t)blockIdx.x, list, n_list, n_query, indptr, qdeg, target_slot, bits_node, bits_query,
                                   sub, (int64_t)0, raw, cols);
}

// ---- small requests: the whole first half of the construction in one block --------------------
// Up to SMALL_E request edges and SMALL_Q queries: the request fits the LDS of one compute unit, and the chain of a
// dozen short kernels above (each 3-10 us whatever its size) becomes one kernel.  Same results, other means:
//   the edges sorted by (node, query) give the candidates in ascending id, the query edges at each, and each
//     target's attached queries in ascending order (the tail of its row);
//   the same radix select on the ratio keys (histogram in LDS);
//   the edges sorted by (query, candidate place) give the query rows in ascending node id.
// No per-node or per-query scratch is touched except the node-to-slot map.  Leaves: cand, qdeg, cand_row, targets,
// target_slot, the nodes' slots, row pointers, work list offsets, the lists of cut rows, the sizes; raw_q = the query rows'
// node ids in row order, raw_t = the request's query indices in (node, query) order, cand_start = where each
// candidate's run starts in raw_t.  k_finish_cols takes the raw rows from there.
// NT threads take up to 2 NT edges, 2 NT queries, 4 NT rows: 1,024 threads in general, 256 for the smallest requests
// (barriers and block-wide sums cost a quarter there).
constexpr int SMALL_E = 2048, SMALL_Q = 2048;
constexpr int SMALL_E_FEW = 512;

// stage barrier of the bitonic network below: stages whose partner distance is at most 64 only move data inside the
// 128 keys a wavefront owns, so wavefront-level ordering is enough there
__device__ inline void sort_stage_sync(bool block_wide) {
    if (block_wide) {
        __syncthreads();
    } else {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
}

// ascending bitonic sort of n2 keys in LDS (n2 a power of two, 128 <= n2 <= 2 * blockDim.x), all threads of the block
template <typename K>
__device__ inline void bitonic_sort_lds(K* key, int n2) {
    const int idx = threadIdx.x;
    for (int k = 2; k <= n2; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            if (idx < (n2 >> 1)) {
                const int i = ((idx & ~(j - 1)) << 1) | (idx & (j - 1));
                const K a = key[i], b = key[i + j];
                const bool up = (i & k) == 0;
                if ((a > b) == up) {
                    key[i] = b;
                    key[i + j] = a;
                }
            }
            // the next stage is (k, j / 2), or (2 k, k) after j == 1
            const int next_j = j > 1 ? (j >> 1) : k;
            sort_stage_sync(j >= 128 || next_j >= 128);
        }
    }
    __syncthreads();
}

template <int NT>
__global__ __launch_bounds__(NT) void k_build_small(
    const int32_t* __restrict__ qe_query, const int32_t* __restrict__ qe_node, int n_e, int n_query, int64_t n_nodes,
    const int64_t* __restrict__ base_indptr, uint32_t gamma_ppm, int n_pass, int lo_final, int part_edges, int policy,
    uint64_t seed, const float* __restrict__ node_scores, DevState* st, HostMailbox* __restrict__ mailbox,
    unsigned long long seq, omg_ctx::NodeRec* __restrict__ node_rec, int32_t* __restrict__ cand, int32_t* __restrict__ qdeg,
    int32_t* __restrict__ cand_row, int32_t* __restrict__ targets, int32_t* __restrict__ target_slot,
    int64_t* __restrict__ indptr, int32_t* __restrict__ part_ptr, int32_t* __restrict__ split_rows,
    int32_t* __restrict__ split_rows_q, int32_t* __restrict__ split_big, int32_t* __restrict__ split_big_q,
    int32_t* __restrict__ raw_q, int32_t* __restrict__ raw_t, int32_t* __restrict__ cand_start) {
    __shared__ uint64_t keyA[SMALL_E];                 // (node << 32) | query, sorted
    __shared__ uint32_t keyB[SMALL_E];                 // (query << 11) | place of the node in R, sorted
    __shared__ uint16_t cstart[SMALL_E + 2];           // first edge of each candidate in keyA
    __shared__ __attribute__((aligned(8))) uint32_t X[SEL_BINS / 2];   // select: histogram, two 16-bit bins per word; later row data
    __shared__ int64_t sh[16];
    __shared__ unsigned long long s_prefix;
    __shared__ long long s_krem;
    __shared__ int s_bad, s_cnt[4];
    const int tid = threadIdx.x;
    BuildCounts* c = &st->counts;
    int n2 = 128;
    while (n2 < n_e) n2 <<= 1;

    // ---- the request, checked
    if (tid == 0) s_bad = 0;
    __syncthreads();
    for (int i = tid; i < n2; i += NT) {
        uint64_t key = ~0ull;
        if (i < n_e) {
            const int32_t q = qe_query[i], u = qe_node[i];
            if (q < 0 || q >= n_query || u < 0 || (int64_t)u >= n_nodes) s_bad = 1;
            else key = ((uint64_t)(uint32_t)u << 32) | (uint32_t)q;
        }
        keyA[i] = key;
    }
    __syncthreads();
    if (s_bad) {                                       // rejected: nothing outside this block has been touched
        if (tid == 0) {
            BuildCounts z{};
            z.err = 1;
            *c = z;
            c->err = 0;                                // the device copy stays clean for the next build
            mailbox->counts = z;
            __threadfence_system();
            __hip_atomic_store(&mailbox->seq, seq, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
        }
        return;
    }
    bitonic_sort_lds(keyA, n2);

    // ---- candidates: runs of equal node in keyA.  Two consecutive edges per thread, so that a block scan numbers them.
    const int i0 = 2 * tid, i1 = 2 * tid + 1;
    const bool h0 = i0 < n_e && (i0 == 0 || (keyA[i0] >> 32) != (keyA[i0 - 1] >> 32));
    const bool h1 = i1 < n_e && (keyA[i1] >> 32) != (keyA[i0] >> 32);
    int64_t total;
    const int before = (int)block_excl_scan((int64_t)h0 + (int64_t)h1, &total, sh);
    const int n_cand = (int)total;
    const int r_e0 = before + (h0 ? 1 : 0) - 1;        // place in R of the node of edge i0 (the run it belongs to)
    const int r_e1 = r_e0 + (h1 ? 1 : 0);
    if (h0) cstart[r_e0] = (uint16_t)i0;
    if (h1) cstart[r_e1] = (uint16_t)i1;
    if (tid == 0) cstart[n_cand] = (uint16_t)n_e;
    for (int i = tid; i < n2; i += NT) keyB[i] = 0xffffffffu;
    __syncthreads();
    if (i0 < n_e) keyB[i0] = ((uint32_t)keyA[i0] << 11) | (uint32_t)r_e0;
    if (i1 < n_e) keyB[i1] = ((uint32_t)keyA[i1] << 11) | (uint32_t)r_e1;
    if (i0 < n_e) raw_t[i0] = (int32_t)(uint32_t)keyA[i0];
    if (i1 < n_e) raw_t[i1] = (int32_t)(uint32_t)keyA[i1];

    // ---- per candidate (two consecutive ones per thread): node, query edges, ranking key
    uint64_t key[2] = {0, 0};
    int64_t deg_b[2] = {0, 0};
    int32_t node[2] = {0, 0}, a_q[2] = {0, 0};
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2) {
        const int r = 2 * tid + s2;
        if (r < n_cand) {
            const int first = cstart[r];
            node[s2] = (int32_t)(keyA[first] >> 32);
            a_q[s2] = (int)cstart[r + 1] - first;
            deg_b[s2] = node_rec[node[s2]].deg;
            key[s2] = policy == OMG_POLICY_RANDOM ? random_key(seed, (uint32_t)node[s2])
                      : policy == OMG_POLICY_SCORE ? score_key(node_scores[node[s2]])
                                                   : ratio_key((uint64_t)a_q[s2], (uint64_t)deg_b[s2]);
            cand[r] = node[s2];
            qdeg[r] = a_q[s2];
            node_rec[node[s2]].slot = r;
            cand_start[r] = first;
        }
    }

    // ---- selection: the same most-significant-digit radix select, histogram in LDS
    const long long k_take = (long long)(((uint64_t)gamma_ppm * (uint64_t)n_cand) / 1000000ull);
    unsigned long long prefix = 0;
    long long k_rem = 0;
    // a handful of candidates: each is ranked against all the others directly (better key first, then smaller id)
    const bool direct = n_cand <= 256;
    bool in_direct[2] = {false, false};
    if (k_take > 0 && direct) {
        uint64_t* kk_l = reinterpret_cast<uint64_t*>(X);
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2)
            if (2 * tid + s2 < n_cand) kk_l[2 * tid + s2] = key[s2] >> lo_final;
        __syncthreads();
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
            const int r = 2 * tid + s2;
            if (r < n_cand) {
                const uint64_t mine = kk_l[r];
                int better = 0;
                for (int j = 0; j < n_cand; ++j) {
                    const uint64_t o = kk_l[j];
                    better += (o > mine || (o == mine && j < r)) ? 1 : 0;
                }
                in_direct[s2] = better < k_take;
            }
        }
        __syncthreads();
    }
    if (k_take > 0 && !direct) {
        constexpr int PER = SEL_BINS / NT;
        k_rem = k_take;
        for (int pass = 0; pass < n_pass; ++pass) {
            const int hi = 64 - SEL_BITS * pass;
            const int lo = hi - SEL_BITS > 0 ? hi - SEL_BITS : 0;
            const int nb = hi - lo;
            const uint64_t dmask = (1ull << nb) - 1;
            for (int i = tid; i < SEL_BINS / 2; i += NT) X[i] = 0;
            __syncthreads();
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2)
                if (2 * tid + s2 < n_cand && (pass == 0 || (key[s2] >> hi) == prefix)) {
                    const uint32_t bin = (uint32_t)((key[s2] >> lo) & dmask);
                    atomicAdd(&X[bin >> 1], 1u << (16 * (bin & 1)));     // a bin holds at most SMALL_E < 2^16
                }
            __syncthreads();
            const int top = SEL_BINS - PER * tid;     // this thread owns bins [top - PER, top), walked downwards
            unsigned int mine[PER];
            int64_t gsum = 0;
#pragma unroll
            for (int j = 0; j < PER; ++j) {
                const int bin = top - 1 - j;
                mine[j] = (X[bin >> 1] >> (16 * (bin & 1))) & 0xffffu;
                gsum += mine[j];
            }
            int64_t tot;
            const int64_t bef = block_excl_scan(gsum, &tot, sh);
            if (bef < k_rem && k_rem <= bef + gsum) {
                int64_t acc = bef;
#pragma unroll
                for (int j = 0; j < PER; ++j) {
                    if (acc + mine[j] >= k_rem) {
                        s_prefix = (pass == 0 ? 0ull : (prefix << nb)) | (unsigned long long)(top - 1 - j);
                        s_krem = k_rem - acc;
                        break;
                    }
                    acc += mine[j];
                }
            }
            __syncthreads();
            prefix = s_prefix;
            k_rem = s_krem;
            __syncthreads();
        }
    }

    // ---- targets in ascending id: above the threshold, plus the first k_rem at it
    uint32_t* tlen_l = X;                              // [SMALL_E] row length of each target (the histogram is done with)
    uint32_t* qlen_l = X + SMALL_E;                    // [SMALL_Q] edges of each query
    uint64_t f[2];
    uint64_t fsum = 0;
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2) {
        f[s2] = 0;
        if (2 * tid + s2 < n_cand && k_take > 0) {
            const uint64_t kk = key[s2] >> lo_final;
            f[s2] = direct ? (in_direct[s2] ? 1ull : 0ull) : kk > prefix ? 1ull : (kk == prefix ? (1ull << 32) : 0ull);
        }
        fsum += f[s2];
    }
    int64_t ftot;
    uint64_t fs = (uint64_t)block_excl_scan((int64_t)fsum, &ftot, sh);
    for (int i = tid; i < SMALL_Q; i += NT) qlen_l[i] = 0;
    int n_target_local = 0;
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2) {
        const int r = 2 * tid + s2;
        if (r < n_cand) {
            const int64_t gt_before = (int64_t)(fs & 0xffffffffull), eq_before = (int64_t)(fs >> 32);
            const bool gt = (f[s2] & 1ull) != 0, eq = (f[s2] >> 32) != 0;
            const bool in_t = gt || (eq && eq_before < k_rem);
            const int64_t t = gt_before + (eq_before < k_rem ? eq_before : k_rem);
            if (in_t) {
                targets[t] = node[s2];
                target_slot[t] = r;
                cand_row[r] = n_query + (int32_t)t;
                tlen_l[t] = (uint32_t)(deg_b[s2] + a_q[s2]);
            } else {
                cand_row[r] = -1;
            }
            if (r == n_cand - 1) n_target_local = (int)t + (in_t ? 1 : 0);
        }
        fs += f[s2];
    }
    if (2 * tid < n_cand && 2 * tid + 2 >= n_cand) s_cnt[0] = n_target_local;       // the thread that owns the last candidate
    if (tid == 0 && n_cand == 0) s_cnt[0] = 0;
    if (tid < 3) s_cnt[1 + tid] = 0;                   // list cursors: cut rows, cut query rows, rows of many parts
    __syncthreads();
    const int n_target = s_cnt[0];
    const int rows_in = n_query + n_target;

    // ---- query rows: edges by (query, place in R); lengths by counting
    if (i0 < n_e) atomicAdd(&qlen_l[(uint32_t)keyA[i0]], 1u);
    if (i1 < n_e) atomicAdd(&qlen_l[(uint32_t)keyA[i1]], 1u);
    bitonic_sort_lds(keyB, n2);                        // (ends with a barrier: the counts above are complete too)
    for (int i = tid; i < n_e; i += NT) raw_q[i] = (int32_t)(keyA[cstart[keyB[i] & 2047u]] >> 32);

    // ---- rows: lengths, parts, their prefix sums; four consecutive rows per thread
    int64_t len[4];
    int np[4];
    int64_t s_len = 0, s_np = 0, s_npq = 0;
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4) {
        const int v = 4 * tid + s4;
        len[s4] = v < n_query ? (int64_t)qlen_l[v] : v < rows_in ? (int64_t)tlen_l[v - n_query] : 0;
        np[s4] = 0;
        if (v < rows_in) {
            const int ps = omg_row_part(len[s4], part_edges);
            np[s4] = (int)((len[s4] + ps - 1) / ps);
            if (np[s4] < 1) np[s4] = 1;
        }
        s_len += len[s4];
        s_np += np[s4];
        if (v < n_query) s_npq += np[s4];
    }
    int64_t nnz, n_parts, n_parts_q;
    int64_t run_len = block_excl_scan(s_len, &nnz, sh);
    int64_t run_np = block_excl_scan(s_np, &n_parts, sh);
    (void)block_excl_scan(s_npq, &n_parts_q, sh);
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4) {
        const int v = 4 * tid + s4;
        if (v < rows_in) {
            indptr[v] = run_len;
            part_ptr[v] = (int32_t)run_np;
        }
        if (v < rows_in && np[s4] > 1) {
            const bool many = np[s4] > OMG_MANY_PARTS;
            if (many) split_big[atomicAdd(&s_cnt[3], 1)] = v;
            else split_rows[atomicAdd(&s_cnt[1], 1)] = v;
        }
        run_len += len[s4];
        run_np += np[s4];
    }
    if (tid == 0) {                                    // the end pointers
        indptr[rows_in] = nnz;
        part_ptr[rows_in] = (int32_t)n_parts;
    }
    __syncthreads();
    // the lists of the query rows (the last layer's) are the query rows of the lists above: a second pass keeps
    // their counters apart
    const int n_split = s_cnt[1], n_many = s_cnt[3];
    __syncthreads();
    if (tid == 0) s_cnt[1] = s_cnt[3] = 0;
    __syncthreads();
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4) {
        const int v = 4 * tid + s4;
        if (v < n_query && np[s4] > 1) {
            if (np[s4] > OMG_MANY_PARTS) split_big_q[atomicAdd(&s_cnt[3], 1)] = v;
            else split_rows_q[atomicAdd(&s_cnt[1], 1)] = v;
        }
    }
    __syncthreads();
    if (tid == 0) {
        BuildCounts z{};
        z.n_cand = n_cand;
        z.n_target = n_target;
        z.nnz_in = nnz;
        z.n_parts = n_parts;
        z.n_parts_last = n_parts_q;
        z.n_split = n_split;
        z.n_split_last = s_cnt[1];
        z.n_split_big = n_many;
        z.n_split_big_last = s_cnt[3];
        *c = z;
        mailbox->counts = z;
        __threadfence_system();
        __hip_atomic_store(&mailbox->seq, seq, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
    }
}

// sorted raw rows -> tagged columns and source degrees; target rows get their base neighbours here.
__device__ inline void tag_source(int32_t src, const omg_ctx::NodeRec* __restrict__ node,
                                  const int32_t* __restrict__ cand_row, const int32_t* __restrict__ qdeg,
                                  int32_t* col, int32_t* deg) {
    const int4 rec = *reinterpret_cast<const int4*>(&node[src]);         // slot and degree: one load
    const int32_t r = rec.x;
    const int32_t row = r >= 0 ? cand_row[r] : -1;
    *col = row >= 0 ? ~row : src;
    *deg = rec.z + (r >= 0 ? qdeg[r] : 0);
}

struct FinishArgs {
    const int64_t* indptr;
    const int32_t* part_ptr;
    int32_t* part_row;              // read here; written by k_finish_small, which makes the work list itself
    int64_t n_parts;
    int part_edges;
    const int32_t *targets, *qdeg, *cand_row;
    const omg_ctx::NodeRec* node;
    const int64_t* base_indptr;
    const int32_t* base_indices;
    int32_t n_query;
    const int32_t *raw_q, *raw_t, *cand_start, *target_slot;
    int32_t *cols, *cdeg;
    int lg_group;
};

// A group of 2^lg_group lanes per work item (row, part), the same cut the aggregation kernels use: every edge is
// a chain of five to seven dependent loads and nothing crosses the lanes, so what counts is how many edges a
// wavefront has in flight; with a wavefront per work item of a dozen edges most lanes idled (a launch took the
// chain's latency times five rounds of wavefronts).  The sorted raw rows are in `cols` itself, or (a small
// request, built by one block) in raw_q / raw_t.  t: the lane's number among all lanes of the launch.
__device__ inline void finish_cols_lane(const FinishArgs& a, int64_t t) {
    const int lane = (int)(t & ((1 << a.lg_group) - 1));
    const int stride = 1 << a.lg_group;
    const int64_t part = t >> a.lg_group;
    if (part >= a.n_parts) return;
    const int v = a.part_row[part];
    const int64_t row_beg = a.indptr[v], row_end = a.indptr[v + 1];
    const int ps = omg_row_part(row_end - row_beg, a.part_edges);
    const int64_t e0 = row_beg + (int64_t)(part - a.part_ptr[v]) * ps;
    const int64_t e1 = e0 + ps < row_end ? e0 + ps : row_end;
    int64_t b0 = 0, dg = 0, tail0 = 0;
    if (v >= a.n_query) {
        const int32_t u = a.targets[v - a.n_query];
        b0 = a.base_indptr[u];
        dg = a.base_indptr[(int64_t)u + 1] - b0;
        if (a.raw_t != nullptr) tail0 = a.cand_start[a.target_slot[v - a.n_query]];
    }
    for (int64_t p = e0 + lane; p < e1; p += stride) {
        int32_t c, d;
        const int64_t j = p - row_beg;
        if (v < a.n_query) {
            tag_source(a.raw_q != nullptr ? a.raw_q[p] : a.cols[p], a.node, a.cand_row, a.qdeg, &c, &d);
        } else if (j < dg) {
            tag_source(a.base_indices[b0 + j], a.node, a.cand_row, a.qdeg, &c, &d);
        } else {
            const int32_t q = a.raw_t != nullptr ? a.raw_t[tail0 + (j - dg)] : a.cols[p];      // sorted query index
            c = ~q;
            d = (int32_t)(a.indptr[q + 1] - a.indptr[q]);
        }
        a.cols[p] = c;
        a.cdeg[p] = d;
    }
}

__global__ __launch_bounds__(TPB) void k_finish_cols(FinishArgs a) { finish_cols_lane(a, gtid()); }

// ---- order of the work items of an inner layer -------------------------------------------------
// Rows hold their sources in ascending id, so the k-th of a row's np parts reads sources from about the
// k/np-th quantile of the table.  Walking the parts phase by phase (phase = the f with ceil(f np / P) <= k <
// ceil((f + 1) np / P)) instead of row by row keeps the wavefronts that run at the same time on the same
// 1/P-th of a table that is larger than the memory-side cache.  With C_f[v] = sum over the rows before v of
// ceil(f np / P) (C_0 = 0, C_P = part_ptr), the parts of phase f in the rows before v number C_{f+1}[v] -
// C_f[v]: one single-block prefix sum over rows gives C_1 .. C_{P-1} (two 32-bit sums per 64-bit word), and
// one thread per part then writes its place.
constexpr int ORDER_WORDS = ORDER_PHASES / 2;            // packed pairs of C_1 .. C_{P-1}

__global__ __launch_bounds__(1024) void k_phase_offsets(const int32_t* __restrict__ part_ptr, int64_t rows_in,
                                                        unsigned long long* __restrict__ row_off /* [(rows_in + 1) x ORDER_WORDS] */) {
    __shared__ int64_t wave_tot[16];
    constexpr int ITEMS = 8;
    unsigned long long carry[ORDER_WORDS];
#pragma unroll
    for (int w = 0; w < ORDER_WORDS; ++w) carry[w] = 0;
    for (int64_t base = 0; base < rows_in + 1; base += 1024 * ITEMS) {
        const int64_t i0 = base + (int64_t)threadIdx.x * ITEMS;
        int np[ITEMS];
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) np[j] = i0 + j < rows_in ? part_ptr[i0 + j + 1] - part_ptr[i0 + j] : 0;
#pragma unroll
        for (int w = 0; w < ORDER_WORDS; ++w) {
            const int f0 = 2 * w + 1, f1 = 2 * w + 2;                       // C_f0 in the low half, C_f1 in the high half
            unsigned long long v[ITEMS], sum = 0;
#pragma unroll
            for (int j = 0; j < ITEMS; ++j) {
                v[j] = (unsigned long long)phase_first(f0, np[j]);
                if (f1 < ORDER_PHASES) v[j] |= (unsigned long long)phase_first(f1, np[j]) << 32;
                sum += v[j];
            }
            int64_t total;
            unsigned long long run = carry[w] + (unsigned long long)block_excl_scan((int64_t)sum, &total, wave_tot);
#pragma unroll
            for (int j = 0; j < ITEMS; ++j) {
                if (i0 + j < rows_in + 1) row_off[(i0 + j) * ORDER_WORDS + w] = run;
                run += v[j];
            }
            carry[w] += (unsigned long long)total;
        }
    }
}

__device__ inline int64_t phase_prefix(const unsigned long long* __restrict__ row_off, int64_t v, int f, int64_t c_last) {
    if (f <= 0) return 0;                                 // C_0
    if (f >= ORDER_PHASES) return c_last;                 // C_P = part_ptr
    const unsigned long long w = row_off[v * ORDER_WORDS + (f - 1) / 2];
    return (int64_t)(((f - 1) & 1) ? (w >> 32) : (w & 0xffffffffull));
}

// place of work item p (the k-th part of row v, which has np parts starting at p0) in the phase order
__device__ inline void write_order(int64_t p, int v, int p0, int np, int64_t rows_in, int64_t n_parts,
                                   const unsigned long long* __restrict__ row_off, int32_t* __restrict__ order) {
    const int k = (int)(p - p0);
    int f = (int)(((int64_t)k * ORDER_PHASES) / np);
    while (f + 1 < ORDER_PHASES && phase_first(f + 1, np) <= k) ++f;         // k in [first(f), first(f + 1))
    while (f > 0 && phase_first(f, np) > k) --f;
    // all parts of the earlier phases = C_f[rows_in]; this phase's parts of the earlier rows = C_{f+1}[v] - C_f[v]
    const int64_t at = phase_prefix(row_off, rows_in, f, n_parts) +
                       (phase_prefix(row_off, v, f + 1, p0) - phase_prefix(row_off, v, f, p0)) + (k - phase_first(f, np));
    order[at] = (int32_t)p;
}

// work item -> its row (binary search in the work list offsets) and, with `order` given, its place in the
// order the inner layers walk the work items in: grouped by the region of the table they read (the k-th of a
// row's np parts reads about the k/np-th quantile, rows being sorted by source id), any order inside a
// region.  Places inside a region come from a cursor: a block counts its items per region in LDS and takes
// that many places with one global atomic per region.  Which place an item gets changes nothing in the
// results (partial sums are indexed by work item, not by place).
__device__ inline void fill_parts_body(int64_t block, const int32_t* __restrict__ part_ptr, int64_t rows_in, int64_t n_parts,
                                       int32_t* __restrict__ part_row, const long long* __restrict__ phase_total,
                                       long long* __restrict__ phase_rank, int32_t* __restrict__ order) {
    __shared__ int l_cnt[ORDER_PHASES];
    __shared__ long long l_base[ORDER_PHASES];
    const int64_t j = block * TPB + threadIdx.x;
    int f = -1, r = 0;
    if (order != nullptr) {
        if (threadIdx.x < ORDER_PHASES) l_cnt[threadIdx.x] = 0;
        __syncthreads();
    }
    if (j < n_parts) {
        int64_t lo = 0, hi = rows_in;                 // last row whose first part is <= j
        while (hi - lo > 1) {
            const int64_t mid = (lo + hi) >> 1;
            if (part_ptr[mid] <= j) lo = mid; else hi = mid;
        }
        part_row[j] = (int32_t)lo;
        if (order != nullptr) {
            const int p0 = part_ptr[lo], np = part_ptr[lo + 1] - p0, k = (int)(j - p0);
            f = (int)(((int64_t)k * ORDER_PHASES) / np);
            while (f + 1 < ORDER_PHASES && phase_first(f + 1, np) <= k) ++f;
            while (f > 0 && phase_first(f, np) > k) --f;
            r = atomicAdd(&l_cnt[f], 1);
        }
    }
    if (order == nullptr) return;
    __syncthreads();
    if (threadIdx.x < ORDER_PHASES) {
        long long before = 0;                         // all items of the earlier regions
        for (int g2 = 0; g2 < (int)threadIdx.x; ++g2) before += phase_total[g2 * 8];
        const int c = l_cnt[threadIdx.x];
        l_base[threadIdx.x] = before + (c ? (long long)atomicAdd((unsigned long long*)&phase_rank[threadIdx.x * 8],
                                                                  (unsigned long long)c) : 0);
    }
    __syncthreads();
    if (f >= 0) order[l_base[f] + r] = (int32_t)j;
}

// The sorts of the rows and the work list need nothing from each other, and each of them is a launch of few blocks
// bound by its chains of barriers or dependent loads: one launch gives every block one of the three jobs (the
// longest-running first), so that their durations overlap instead of adding up.
struct SortFillArgs {
    int64_t nb_radix, nb_wave;                  // blocks that sort a medium segment or a piece; blocks of short segments
    const int32_t *list_med, *list_small;
    int64_t n_med, n_small, n_sub;
    int32_t n_query;
    const int64_t* indptr;
    const int32_t *qdeg, *target_slot;
    int bits_node, bits_query;
    SubSeg* sub;
    int32_t *raw, *cols;
    const int32_t* part_ptr;
    int64_t rows_in, n_parts;
    int32_t* part_row;
    const long long* phase_total;
    long long* phase_rank;
    int32_t* order;
};

// RADIX = false: a batch without medium or long rows; the launch then does not carry the radix sort's 32 KB of LDS,
// which would hold the blocks of the other two jobs to five per compute unit.
template <bool RADIX>
__global__ __launch_bounds__(TPB) void k_sort_fill(SortFillArgs a) {
    int64_t b = (int64_t)blockIdx.x;
    if constexpr (RADIX) {
        if (b < a.nb_radix) {
            segsort_radix_body<TPB, false>(b, a.list_med, a.n_med, a.n_query, a.indptr, a.qdeg, a.target_slot, a.bits_node,
                                           a.bits_query, a.sub, a.n_sub, a.raw, a.cols);
            return;
        }
        b -= a.nb_radix;
    }
    if (b < a.nb_wave) {
        segsort_wave_body(b, a.list_small, a.n_small, a.n_query, a.indptr, a.qdeg, a.target_slot, a.raw, a.cols);
        return;
    }
    b -= a.nb_wave;
    fill_parts_body(b, a.part_ptr, a.rows_in, a.n_parts, a.part_row, a.phase_total, a.phase_rank, a.order);
}

__global__ void k_fill_order(const int32_t* __restrict__ part_ptr, const int32_t* __restrict__ part_row, int64_t rows_in,
                             int64_t n_parts, const unsigned long long* __restrict__ row_off, int32_t* __restrict__ order) {
    const int64_t p = gtid();
    if (p >= n_parts) return;
    const int v = part_row[p];
    const int p0 = part_ptr[v];
    write_order(p, v, p0, part_ptr[v + 1] - p0, rows_in, n_parts, row_off, order);
}

__global__ void k_clear_slots(const int32_t* __restrict__ cand, BuildCounts* c, int64_t n_max,
                              omg_ctx::NodeRec* __restrict__ node) {
    const int64_t r = gtid();
    if (r == 0) c->err = 0;                       // the host has read the counters of this build already
    if (r >= n_max || r >= c->n_cand) return;
    node[cand[r]].slot = -1;
}

// The second half of the construction for a request of a few thousand edges, in one block: the work list, then
// the tagged columns, then the nodes' slots back to -1 (three launches of a few microseconds each otherwise, and
// such a batch's time is its launches).  The steps are separated by block barriers: each reads what all threads of
// the step before have written.
__global__ __launch_bounds__(1024) void k_finish_small(FinishArgs a, int64_t rows_in, const int32_t* __restrict__ cand,
                                                       BuildCounts* c, int64_t n_max, omg_ctx::NodeRec* __restrict__ node) {
    for (int64_t j = threadIdx.x; j < a.n_parts; j += 1024) {
        int64_t lo = 0, hi = rows_in;                 // last row whose first part is <= j
        while (hi - lo > 1) {
            const int64_t mid = (lo + hi) >> 1;
            if (a.part_ptr[mid] <= j) lo = mid; else hi = mid;
        }
        a.part_row[j] = (int32_t)lo;
    }
    __syncthreads();
    const int64_t lanes = a.n_parts << a.lg_group;
    for (int64_t t = threadIdx.x; t < lanes; t += 1024) finish_cols_lane(a, t);
    __syncthreads();
    const int64_t n_cand = c->n_cand < n_max ? c->n_cand : n_max;
    for (int64_t r = threadIdx.x; r < n_cand; r += 1024) node[cand[r]].slot = -1;
    if (threadIdx.x == 0) c->err = 0;                 // the host has read the counters of this build already
}

__global__ void k_check_indptr(const int64_t* __restrict__ indptr, int64_t n, BuildCounts* c) {
    const int64_t i = gtid();
    if (i >= n) return;
    const int64_t a = indptr[i], b = indptr[i + 1];
    if ((i == 0 && a != 0) || b < a || b - a >= ((int64_t)1 << 31)) atomicOr(&c->err, 1);
    else atomicMax((unsigned long long*)&c->n_parts, (unsigned long long)(b - a));   // largest degree
    if (i == n - 1) c->nnz_in = b;
}

__global__ void k_check_indices(const int32_t* __restrict__ indices, int64_t nnz, int64_t n, int64_t per_thread,
                                BuildCounts* c) {
    const int64_t t = gtid();
    bool bad = false;
    for (int64_t j = 0; j < per_thread; ++j) {          // strided so that a wavefront reads consecutive entries
        const int64_t e = (t / 64) * 64 * per_thread + j * 64 + (t % 64);
        if (e < nnz) {
            const int32_t u = indices[e];
            bad |= (u < 0 || (int64_t)u >= n);
        }
    }
    if (bad) atomicOr(&c->err, 1);
}

// every node's record between builds: no slot, nothing counted, its degree in the training graph
__global__ void k_init_nodes(omg_ctx::NodeRec* __restrict__ node, const int64_t* __restrict__ base_indptr, int64_t n) {
    const int64_t u = gtid();
    if (u >= n) return;
    *reinterpret_cast<int4*>(&node[u]) = make_int4(-1, 0, (int)(base_indptr[u + 1] - base_indptr[u]), 0);
}

// The host's wait for the sizes of build number `seq`: it polls the pinned mailbox.  Should the number not appear (a
// kernel failed, or the queue was not submitted), it falls back to waiting for the stream.
int wait_for_sizes(omg_ctx* ctx, unsigned long long seq) {
    const auto t0 = std::chrono::steady_clock::now();
    for (unsigned spin = 0;; ++spin) {
        if (__atomic_load_n(&ctx->mailbox->seq, __ATOMIC_ACQUIRE) == seq) return OMG_OK;
        if ((spin & 1023u) == 1023u &&
            std::chrono::duration_cast<std::chrono::milliseconds>(std::chrono::steady_clock::now() - t0).count() >= 20) break;
    }
    OMG_HIP(hipStreamSynchronize(ctx->stream));
    return __atomic_load_n(&ctx->mailbox->seq, __ATOMIC_ACQUIRE) == seq ? OMG_OK : OMG_EHIP;
}

int bits_for(uint64_t max_value) {
    int b = 1;
    while (b < 64 && (max_value >> b) != 0) ++b;
    return b;
}

}  // namespace

int omg_init_state(omg_ctx* ctx) {
    const int64_t n = ctx->base.n_nodes;
    const int64_t n_words = (n + 31) / 32;
    OMG_TRY(ctx->devState.ensure(sizeof(DevState)));
    OMG_TRY(ctx->bitmap.ensure(sizeof(uint32_t) * (size_t)(n_words + 1)));
    OMG_HIP(hipMemsetAsync(ctx->devState.p, 0, sizeof(DevState), ctx->stream));
    OMG_HIP(hipMemsetAsync(ctx->bitmap.p, 0, sizeof(uint32_t) * (size_t)(n_words + 1), ctx->stream));
    if (n_words > TWO_LEVEL_WORDS) {
        const int64_t n_words1 = (n_words + 31) / 32;
        OMG_TRY(ctx->bitmap1.ensure(sizeof(uint32_t) * (size_t)(n_words1 + 1)));
        OMG_HIP(hipMemsetAsync(ctx->bitmap1.p, 0, sizeof(uint32_t) * (size_t)(n_words1 + 1), ctx->stream));
    }
    ctx->counts_dev = &static_cast<DevState*>(ctx->devState.p)->counts;
    hipLaunchKernelGGL(k_init_nodes, dim3(grid_for(n)), dim3(TPB), 0, ctx->stream, ctx->node, ctx->base.indptr, n);
    OMG_HIP(hipGetLastError());
    return OMG_OK;
}

// One pass over the training graph when a context is created: row pointers start at zero and never
// decrease, every degree fits 31 bits, every neighbour id is a node.  The kernels rely on this.
int omg_validate_base(omg_ctx* ctx) {
    hipStream_t s = ctx->stream;
    const int64_t n = ctx->base.n_nodes;
    OMG_HIP(hipMemsetAsync(ctx->counts_dev, 0, sizeof(BuildCounts), s));
    hipLaunchKernelGGL(k_check_indptr, dim3(grid_for(n)), dim3(TPB), 0, s, ctx->base.indptr, n, ctx->counts_dev);
    OMG_HIP(hipMemcpyAsync(ctx->counts_host, ctx->counts_dev, sizeof(BuildCounts), hipMemcpyDeviceToHost, s));
    OMG_HIP(hipStreamSynchronize(s));
    if (ctx->counts_host->err != 0) return OMG_EINVAL;
    const int64_t nnz = ctx->counts_host->nnz_in;
    ctx->max_base_deg = ctx->counts_host->n_parts;
    if (nnz > 0) {
        if (ctx->base.indices == nullptr) return OMG_EINVAL;
        const int64_t per_thread = 16;
        hipLaunchKernelGGL(k_check_indices, dim3(grid_for((nnz + per_thread - 1) / per_thread)), dim3(TPB), 0, s,
                           ctx->base.indices, nnz, n, per_thread, ctx->counts_dev);
        OMG_HIP(hipMemcpyAsync(ctx->counts_host, ctx->counts_dev, sizeof(BuildCounts), hipMemcpyDeviceToHost, s));
        OMG_HIP(hipStreamSynchronize(s));
        if (ctx->counts_host->err != 0) return OMG_ERANGE;
    }
    return OMG_OK;
}

int omg_graph_order(omg_ctx* ctx, omg_graph* g) {
    if (g->order_ready) return OMG_OK;
    if (g->c.n_parts <= 0 || g->c.n_parts >= ((int64_t)1 << 31)) return OMG_EUNSUPPORTED;
    hipStream_t s = ctx->stream;
    OMG_TRY(ctx->rowOff.ensure(sizeof(unsigned long long) * (size_t)(g->rows_in + 2) * ORDER_WORDS));
    OMG_TRY(g->order.ensure(sizeof(int32_t) * (size_t)(g->c.n_parts + 1)));
    hipLaunchKernelGGL(k_phase_offsets, dim3(1), dim3(1024), 0, s, g->part_ptr.as<int32_t>(), g->rows_in,
                       ctx->rowOff.as<unsigned long long>());
    hipLaunchKernelGGL(k_fill_order, dim3(grid_for(g->c.n_parts)), dim3(TPB), 0, s, g->part_ptr.as<int32_t>(),
                       g->part_row.as<int32_t>(), g->rows_in, g->c.n_parts, ctx->rowOff.as<unsigned long long>(),
                       g->order.as<int32_t>());
    OMG_HIP(hipGetLastError());
    g->order_ready = true;
    return OMG_OK;
}

static int build_body(omg_ctx* ctx, omg_graph* g, int32_t n_query, int64_t n_e, const int32_t* qe_query,
                      const omg_node_t* qe_node, uint32_t gamma_ppm, const omg_node_t* rset, int64_t n_rset) {
    hipStream_t s = ctx->stream;
    const int64_t n_nodes = ctx->base.n_nodes;
    const int64_t n_words = (n_nodes + 31) / 32;
    const int64_t max_cand = n_e < n_nodes ? n_e : n_nodes;        // upper bound of |R| and of |T|
    // Every ratio has a denominator below 2^m (m from the largest base degree plus the number of
    // request edges), so the top 2m bits of the 64-bit keys order them exactly.
    const int m_bits = bits_for((uint64_t)ctx->max_base_deg + (uint64_t)n_e);
    const int sel_bits = ctx->policy == OMG_POLICY_RANDOM ? 39 : ctx->policy == OMG_POLICY_SCORE ? 32
                         : (2 * m_bits < 64 ? 2 * m_bits : 64);
    const int n_pass = (sel_bits + SEL_BITS - 1) / SEL_BITS;
    const int lo_final = 64 - SEL_BITS * n_pass > 0 ? 64 - SEL_BITS * n_pass : 0;
    const bool lds_q = n_query <= LDS_QUERY_MAX;
    const size_t lds_bytes = lds_q ? sizeof(int32_t) * (size_t)(n_query > 0 ? n_query : 1) : 0;
    g->built = false;
    g->order_ready = false;
    g->n_query = n_query;
    g->n_qedges = n_e;
    if (n_e == 0 && rset != nullptr && n_rset > 0) return OMG_ERANGE;     // no candidates to choose from
    // work items of at most part_edges edges: small batches get smaller parts so that the last layer
    // (the request's edges only) still spreads over the whole chip.  The attention kernel stages a work
    // item's scores and merges cut rows by rescaling, which costs more per work item: its caller asks for
    // at least 64 edges, so that most rows stay whole.
    int part_edges = OMG_PART_EDGES;
    int min_part = ctx->hint_min_part_edges > 32 ? ctx->hint_min_part_edges : 32;
    // many short query rows (at least 8,192 of them, 64 edges or fewer on average): 64-edge work items keep
    // most rows whole (no partial sums, no combine) and the rows alone still fill the chip
    if (n_query >= 8192 && n_e / n_query <= 64) min_part = min_part > 64 ? min_part : 64;
    // a request of a few thousand edges cannot fill the chip whatever the part size: rows of up to 64 edges stay
    // whole there (one launch less per layer for the batches whose time is all launches)
    if (n_e <= 4096) min_part = min_part > 64 ? min_part : 64;
    // rows of 2 KB and more read once each from a table far beyond the caches: a work item's partial sums are as
    // wide as two of the rows it reads, and the launch that adds them up costs as much again; with 64 edges per
    // work item half as many are written (2 KB rows of a 61 GB table: aggregation 0.622 -> 0.599 ms).  Where the
    // rows are read several times over (2.4 KB rows of a 0.55 GB table) the gather itself is 2.5 % slower with 64.
    if (ctx->hint_row_bytes >= 2048 && ctx->hint_table_bytes > ((int64_t)8 << 30)) min_part = min_part > 64 ? min_part : 64;
    while (part_edges > min_part && n_e / part_edges < 8192) part_edges >>= 1;
    g->part_edges = part_edges;

    // ---- every allocation that does not depend on the batch's content, before any launch
    // rows: the queries and at most as many targets as the budget (or the given set) allows
    const int64_t max_target = rset != nullptr ? n_rset : (int64_t)(((uint64_t)gamma_ppm * (uint64_t)max_cand) / 1000000ull);
    const int64_t n_rows_b = (int64_t)n_query + max_target + 1;      // upper bound of rows_in, plus the end-pointer entry
    const size_t nc = (size_t)max_cand, ns = (size_t)n_rows_b + 1;
    OMG_TRY(g->indptr.ensure(sizeof(int64_t) * ns));
    OMG_TRY(g->part_ptr.ensure(sizeof(int32_t) * ns));
    OMG_TRY(g->split_rows.ensure(sizeof(int32_t) * ns));
    OMG_TRY(g->split_rows_q.ensure(sizeof(int32_t) * (size_t)(n_query + 2)));
    OMG_TRY(g->split_big.ensure(sizeof(int32_t) * ns));
    OMG_TRY(g->split_big_q.ensure(sizeof(int32_t) * (size_t)(n_query + 2)));
    OMG_TRY(g->cand.ensure(sizeof(int32_t) * (nc + 1)));
    OMG_TRY(g->qdeg.ensure(sizeof(int32_t) * (nc + 1)));
    OMG_TRY(g->cand_row.ensure(sizeof(int32_t) * (nc + 1)));
    OMG_TRY(g->targets.ensure(sizeof(int32_t) * (nc + 1)));
    OMG_TRY(g->target_slot.ensure(sizeof(int32_t) * (nc + 1)));
    // per-query counters and cursors are all zero between builds; a fresh allocation is cleared once
    const size_t q_bytes = sizeof(int32_t) * (size_t)(n_query + 2);
    for (DevBuf* b : {&ctx->qcnt, &ctx->qcur})
        if (q_bytes > b->cap) {
            OMG_TRY(b->ensure(q_bytes));
            OMG_HIP(hipMemsetAsync(b->p, 0, b->cap, s));
        }
    OMG_TRY(ctx->tcur.ensure(sizeof(int32_t) * (nc + 1)));
    OMG_TRY(ctx->skey.ensure(sizeof(uint64_t) * (nc + 1)));
    OMG_TRY(ctx->flag.ensure(sizeof(uint64_t) * (nc + 1)));
    OMG_TRY(ctx->tLen.ensure(sizeof(int64_t) * (nc + 2)));
    OMG_TRY(ctx->tOff.ensure(sizeof(int64_t) * (ns + 64)));     // row lengths before the prefix sum
    OMG_TRY(ctx->nParts.ensure(sizeof(int32_t) * (ns + 64)));
    OMG_TRY(ctx->listSmall.ensure(sizeof(int32_t) * ns));
    OMG_TRY(ctx->listMed.ensure(sizeof(int32_t) * ns));
    OMG_TRY(ctx->listBig.ensure(sizeof(int32_t) * ns));
    const bool two_level = n_words > TWO_LEVEL_WORDS;
    const int64_t n_words1 = (n_words + 31) / 32;
    const int64_t max_touched = n_e < n_words ? n_e : n_words;      // upper bound of the words that hold a candidate
    // totals of chunks / blocks for the prefix sums that their consumers finish themselves
    const int fused_max = ctx->fused_sum_max;
    const int64_t n_chunks_words = ((two_level ? n_words1 : n_words) + 63) / 64;
    const int64_t n_chunks_touched = two_level ? (max_touched + 63) / 64 + 1 : 0;
    const int64_t n_flag_blocks = (max_cand + SUM_BLOCK) / SUM_BLOCK;
    const int64_t n_row_blocks = (n_rows_b + SUM_BLOCK - 1) / SUM_BLOCK;
    OMG_TRY(ctx->chunkTot.ensure(sizeof(int32_t) * (size_t)(n_chunks_words + n_chunks_touched + 4)));
    OMG_TRY(ctx->flagTot.ensure(sizeof(uint64_t) * (size_t)(n_flag_blocks + 2)));
    OMG_TRY(ctx->rowTot.ensure(sizeof(int64_t) * 2 * (size_t)(n_row_blocks + 2)));
    if (two_level) {
        OMG_TRY(ctx->wordList.ensure(sizeof(int32_t) * (size_t)(max_touched + 1)));
        OMG_TRY(ctx->wordCnt.ensure(sizeof(int32_t) * (size_t)(max_touched + 2)));
    }

    DevState* st = static_cast<DevState*>(ctx->devState.p);
    BuildCounts* cd = &st->counts;
    uint32_t* bitmap = ctx->bitmap.as<uint32_t>();
    uint32_t* bitmap1 = two_level ? ctx->bitmap1.as<uint32_t>() : nullptr;
    int32_t* qcnt = ctx->qcnt.as<int32_t>();
    int32_t* qcur = ctx->qcur.as<int32_t>();
    int32_t* tcur = ctx->tcur.as<int32_t>();
    uint64_t* skey = ctx->skey.as<uint64_t>();
    uint64_t* flag = ctx->flag.as<uint64_t>();
    uint64_t* flag_tot = ctx->flagTot.as<uint64_t>();
    int64_t* tot_len = ctx->rowTot.as<int64_t>();
    int64_t* tot_np = tot_len + n_row_blocks + 2;
    int32_t* chunk_tot = ctx->chunkTot.as<int32_t>();
    int32_t* chunk_tot2 = chunk_tot + n_chunks_words + 2;          // touched words (large graphs)
    int64_t* tlen = ctx->tLen.as<int64_t>();
    int64_t* rowlen = ctx->tOff.as<int64_t>();
    int32_t* nparts = ctx->nParts.as<int32_t>();
    int32_t* list_small = ctx->listSmall.as<int32_t>();
    int32_t* list_med = ctx->listMed.as<int32_t>();
    int32_t* list_big = ctx->listBig.as<int32_t>();
    const int bn = bits_for((uint64_t)n_nodes - 1);
    const int bq = bits_for((uint64_t)(n_query > 0 ? n_query - 1 : 0));
    int32_t* cand = g->cand.as<int32_t>();
    int32_t* qdeg = g->qdeg.as<int32_t>();
    int32_t* cand_row = g->cand_row.as<int32_t>();
    int32_t* targets = g->targets.as<int32_t>();
    int32_t* target_slot = g->target_slot.as<int32_t>();
    int64_t* indptr = g->indptr.as<int64_t>();
    int32_t* part_ptr = g->part_ptr.as<int32_t>();
    const int e_items = edge_items(n_e);
    const int e_block = n_e <= 65536 ? 256 : EDGE_BLOCK;          // small requests: smaller blocks, more of them
    const unsigned ge = grid_for(n_e, (int64_t)e_block * e_items);
    const unsigned gc = grid_for(max_cand + 1);
    // totals beyond what a consumer's block can add up by itself are first turned into prefixes by one block
    auto totals_to_prefixes = [&](auto* tot, int64_t n_tot) -> int {
        if (n_tot <= fused_max) return 0;
        using T = std::remove_pointer_t<decltype(tot)>;
        hipLaunchKernelGGL((k_scan_block<PtrLoad<T>, T>), dim3(1), dim3(1024), 0, s, PtrLoad<T>{tot}, tot, n_tot);
        return 1;
    };

    // a request that fits the LDS of one compute unit: the whole first half in one block
    const bool small = ctx->small_path && rset == nullptr && n_e > 0 && n_e <= SMALL_E && n_query <= SMALL_Q;
    const unsigned long long want_seq = ++ctx->build_seq;
    int32_t *raw_q = nullptr, *raw_t = nullptr;
    if (small) {
        OMG_TRY(ctx->smallRaw.ensure(sizeof(int32_t) * 2 * SMALL_E));
        raw_q = ctx->smallRaw.as<int32_t>();
        raw_t = raw_q + SMALL_E;
        ctx->slots_dirty = true;
#define OMG_LAUNCH_SMALL(NT)                                                                                             \
    hipLaunchKernelGGL(k_build_small<NT>, dim3(1), dim3(NT), 0, s, qe_query, qe_node, (int)n_e, (int)n_query, n_nodes,       \
                       ctx->base.indptr, gamma_ppm, n_pass, lo_final, part_edges, ctx->policy, ctx->policy_seed,            \
                       ctx->node_scores, st, ctx->mailbox_dev, want_seq, ctx->node, cand, qdeg, cand_row, targets,     \
                       target_slot, indptr, part_ptr, g->split_rows.as<int32_t>(), g->split_rows_q.as<int32_t>(),           \
                       g->split_big.as<int32_t>(), g->split_big_q.as<int32_t>(), raw_q, raw_t, tcur)
        if (n_e <= SMALL_E_FEW && n_query <= SMALL_E_FEW) OMG_LAUNCH_SMALL(256);
        else OMG_LAUNCH_SMALL(1024);
#undef OMG_LAUNCH_SMALL
    } else {
    if (n_e > 0) {
    // how the request edges at a node are counted (see k_count): by the bitmap first when the request has fewer than
    // one edge per 8 nodes of the graph
    const int bit_first = n_e * 8 < n_nodes ? 1 : 0;
#define OMG_LAUNCH_COUNT(LDSQ, ITEMS)                                                                                      \
    do {                                                                                                                   \
        if (bit_first)                                                                                                     \
            hipLaunchKernelGGL((k_count<LDSQ, ITEMS, true>), dim3(ge), dim3(e_block), LDSQ ? lds_bytes : 0, s, qe_query,   \
                               qe_node, n_e, n_query, n_nodes, qcnt, ctx->node, bitmap, bitmap1, cd);                     \
        else                                                                                                               \
            hipLaunchKernelGGL((k_count<LDSQ, ITEMS, false>), dim3(ge), dim3(e_block), LDSQ ? lds_bytes : 0, s, qe_query,  \
                               qe_node, n_e, n_query, n_nodes, qcnt, ctx->node, bitmap, bitmap1, cd);                     \
    } while (0)
        if (lds_q) {
            if (e_items == 1) OMG_LAUNCH_COUNT(true, 1);
            else if (e_items == 2) OMG_LAUNCH_COUNT(true, 2);
            else OMG_LAUNCH_COUNT(true, 4);
        } else {
            if (e_items == 1) OMG_LAUNCH_COUNT(false, 1);
            else if (e_items == 2) OMG_LAUNCH_COUNT(false, 2);
            else OMG_LAUNCH_COUNT(false, 4);
        }
#undef OMG_LAUNCH_COUNT
        // candidates in ascending id
        if (!two_level) {
            hipLaunchKernelGGL(k_popc_chunks, dim3(grid_for(n_words, 1024)), dim3(1024), 0, s, (const uint32_t*)bitmap, n_words,
                               chunk_tot);
            const int scanned = totals_to_prefixes(chunk_tot, n_chunks_words);
            ctx->slots_dirty = true;
            hipLaunchKernelGGL(k_emit_candidates, dim3(grid_for(4 * n_words)), dim3(TPB), 0, s, bitmap,
                               (const int32_t*)chunk_tot, scanned, n_words, (const int32_t*)nullptr, (const DevState*)st,
                               ctx->node, cand, qdeg, skey, cd, ctx->policy,
                               ctx->policy_seed, ctx->node_scores, bit_first);
        } else {
            int32_t* word_list = ctx->wordList.as<int32_t>();
            int32_t* word_cnt = ctx->wordCnt.as<int32_t>();
            hipLaunchKernelGGL(k_popc_chunks, dim3(grid_for(n_words1, 1024)), dim3(1024), 0, s, (const uint32_t*)bitmap1,
                               n_words1, chunk_tot);
            const int scanned1 = totals_to_prefixes(chunk_tot, n_chunks_words);
            hipLaunchKernelGGL(k_list_words, dim3(grid_for(n_words1)), dim3(TPB), 0, s, bitmap1,
                               (const int32_t*)chunk_tot, scanned1, n_words1, (const uint32_t*)bitmap, word_list, word_cnt, st);
            hipLaunchKernelGGL(k_list_chunks, dim3(grid_for(max_touched + 64, 1024)), dim3(1024), 0, s,
                               (const int32_t*)word_cnt, (const DevState*)st, max_touched, chunk_tot2);
            const int scanned2 = totals_to_prefixes(chunk_tot2, n_chunks_touched);
            ctx->slots_dirty = true;
            hipLaunchKernelGGL(k_emit_candidates, dim3(grid_for(4 * max_touched)), dim3(TPB), 0, s, bitmap,
                               (const int32_t*)chunk_tot2, scanned2, max_touched,
                               (const int32_t*)word_list, (const DevState*)st, ctx->node,
                               cand, qdeg, skey, cd, ctx->policy, ctx->policy_seed, ctx->node_scores, bit_first);
        }
        // selection
        const unsigned gf = (unsigned)n_flag_blocks;
        if (rset == nullptr) {
            if (gamma_ppm > 0) {
                if (max_cand <= SELECT_ONE_BLOCK_MAX) {
                    // (max_cand bounds the number of candidates: keys per thread from it)
                    if (max_cand <= 8 * 1024)
                        hipLaunchKernelGGL(k_select_all<8>, dim3(1), dim3(1024), 0, s, (const uint64_t*)skey, st, n_pass, gamma_ppm);
                    else if (max_cand <= 16 * 1024)
                        hipLaunchKernelGGL(k_select_all<16>, dim3(1), dim3(1024), 0, s, (const uint64_t*)skey, st, n_pass, gamma_ppm);
                    else if (max_cand <= 32 * 1024)
                        hipLaunchKernelGGL(k_select_all<32>, dim3(1), dim3(1024), 0, s, (const uint64_t*)skey, st, n_pass, gamma_ppm);
                    else
                        hipLaunchKernelGGL(k_select_all<0>, dim3(1), dim3(1024), 0, s, (const uint64_t*)skey, st, n_pass, gamma_ppm);
                } else {
                    const dim3 gs(grid_for(max_cand, 1024 * SEL_ITEMS));
                    hipLaunchKernelGGL(k_select_hist, gs, dim3(1024), 0, s, skey, st, 0);
                    hipLaunchKernelGGL(k_select_find, dim3(1), dim3(1024), 0, s, st, 0, gamma_ppm);
                    if (n_pass > 1) {
                        // (the flags are written after the select: until then their buffer holds the list)
                        hipLaunchKernelGGL(k_select_compact, gs, dim3(1024), 0, s, (const uint64_t*)skey, st, flag);
                        hipLaunchKernelGGL(k_select_rest, dim3(1), dim3(1024), 0, s, (const uint64_t*)flag, st, n_pass, lo_final);
                    }
                }
            }
            hipLaunchKernelGGL(k_flag, dim3(gf), dim3(SUM_BLOCK), 0, s, skey, st, lo_final, gamma_ppm == 0 ? 1 : 0, max_cand,
                               flag, flag_tot);
        } else {
            hipLaunchKernelGGL(k_zero_flags, dim3(gc), dim3(TPB), 0, s, st, max_cand, flag);
            if (n_rset > 0)
                hipLaunchKernelGGL(k_mark_given, dim3(grid_for(n_rset)), dim3(TPB), 0, s, rset, n_rset, n_nodes,
                                   ctx->node, flag, cd);
            hipLaunchKernelGGL(k_flag_totals, dim3(gf), dim3(SUM_BLOCK), 0, s, (const uint64_t*)flag, max_cand, flag_tot);
        }
        const int scanned_f = totals_to_prefixes(flag_tot, n_flag_blocks);
        hipLaunchKernelGGL(k_targets, dim3(gf), dim3(SUM_BLOCK), 0, s, cand, qdeg, (const uint64_t*)flag,
                           (const uint64_t*)flag_tot, scanned_f, st, n_query, ctx->base.indptr, targets, target_slot,
                           cand_row, tcur, tlen);
    } else {
        OMG_HIP(hipMemsetAsync(st, 0, offsetof(DevState, hist), s));      // no edges: nothing else resets the counters
    }
    hipLaunchKernelGGL(k_rowlen, dim3((unsigned)n_row_blocks), dim3(SUM_BLOCK), 0, s, qcnt, qcur, tlen, qdeg, target_slot,
                       n_query, n_rows_b, part_edges, cd, rowlen, nparts, tot_len, tot_np, list_small, list_med, list_big,
                       g->split_rows.as<int32_t>(), g->split_rows_q.as<int32_t>(), g->split_big.as<int32_t>(),
                       g->split_big_q.as<int32_t>(), st->phase_total);
    int scanned_r = 0;
    if (n_row_blocks > fused_max) {
        totals_to_prefixes(tot_len, n_row_blocks);
        scanned_r = totals_to_prefixes(tot_np, n_row_blocks);
    }
    // the sizes go to the host with this kernel (pinned memory): no copy, and no event to sleep on
    // Work the caller wants done as soon as the targets are known (the layer-0 buffer) rides in the same launch:
    // it keeps the GPU busy while the host reads the sizes and launches again.
    InitBufferArgs init{};
    int64_t n_init_blocks = 0;
    if (ctx->early.armed && ctx->early.max_rows > 0) {
        const omg_table* f = ctx->early.features;
        init = InitBufferArgs{f->data, f->dtype, f->ld, f->dim, ctx->early.query_feats, ctx->early.ld_q, targets, n_query,
                              ctx->early.max_rows, (const BuildCounts*)cd, ctx->early.buf0, ctx->early.ld0};
        constexpr int64_t PER = SUM_BLOCK / 128;
        n_init_blocks = (ctx->early.max_rows + PER - 1) / PER;
        if (n_init_blocks > 2048) n_init_blocks = 2048;
    }
    hipLaunchKernelGGL(k_rowptr, dim3((unsigned)(n_row_blocks + n_init_blocks)), dim3(SUM_BLOCK), 0, s, (const int64_t*)rowlen,
                       (const int32_t*)nparts, n_rows_b, (const int64_t*)tot_len, (const int64_t*)tot_np, scanned_r, indptr,
                       part_ptr, (const BuildCounts*)cd, ctx->mailbox_dev, want_seq, (int)n_row_blocks, init);
    if (ctx->early.armed) ctx->early.done = true;
    }
    OMG_HIP(hipGetLastError());

    if (ctx->early.armed && !ctx->early.done) {
        // (a small request: its one kernel has left the targets)
        OMG_TRY(omg_launch_init_buffer_dev(ctx->early.features, ctx->early.query_feats, ctx->early.ld_q, targets, n_query, cd,
                                           ctx->early.max_rows, ctx->early.buf0, ctx->early.ld0, s));
        ctx->early.done = true;
    }
    OMG_TRY(wait_for_sizes(ctx, want_seq));
    g->c = *ctx->counts_host;
    g->rows_in = n_query + g->c.n_target;

    if (g->c.err != 0) return OMG_ERANGE;              // the caller of this function returns the node slots to -1

    // ---- columns and work list, now that their sizes are known
    OMG_TRY(g->cols.ensure(sizeof(int32_t) * (size_t)(g->c.nnz_in + 1)));
    OMG_TRY(g->cdeg.ensure(sizeof(int32_t) * (size_t)(g->c.nnz_in + 1)));
    OMG_TRY(g->part_row.ensure(sizeof(int32_t) * (size_t)(g->c.n_parts + 1)));
    OMG_TRY(ctx->sortTmp.ensure(sizeof(int32_t) * (size_t)(g->c.nnz_in + 1)));
    OMG_TRY(ctx->subSeg.ensure(sizeof(SubSeg) * (size_t)(16 * g->c.n_big + 1)));
    int32_t* cols = g->cols.as<int32_t>();
    int32_t* raw = ctx->sortTmp.as<int32_t>();
    if (n_e > 0 && !small) {
#define OMG_LAUNCH_BUCKET(LDSQ, ITEMS)                                                                                   \
    hipLaunchKernelGGL((k_bucket<LDSQ, ITEMS>), dim3(ge), dim3(e_block), LDSQ ? lds_bytes : 0, s, qe_query, qe_node, n_e, \
                       indptr, ctx->node, cand_row, qcur, tcur, n_query, raw)
        if (lds_q) {
            if (e_items == 1) OMG_LAUNCH_BUCKET(true, 1);
            else if (e_items == 2) OMG_LAUNCH_BUCKET(true, 2);
            else OMG_LAUNCH_BUCKET(true, 4);
        } else {
            if (e_items == 1) OMG_LAUNCH_BUCKET(false, 1);
            else if (e_items == 2) OMG_LAUNCH_BUCKET(false, 2);
            else OMG_LAUNCH_BUCKET(false, 4);
        }
#undef OMG_LAUNCH_BUCKET
    }
    // rows of more than SORT_MED_MAX keys are cut into 16 pieces by their top bits first
    const bool sorts = n_e > 0 && !small;
    const int64_t n_sub = sorts ? 16 * g->c.n_big : 0;
    SubSeg* sub = ctx->subSeg.as<SubSeg>();
    if (sorts && g->c.n_big > 0)
        hipLaunchKernelGGL(k_segsort_split, dim3((unsigned)g->c.n_big), dim3(1024), 0, s, list_big, g->c.n_big, n_query,
                           indptr, qdeg, target_slot, bn, bq, sub, raw, cols);
    // tagging the columns: lanes per work item = the power of two at or above the average number of edges, 8 .. 64
    FinishArgs fa{};
    fa.indptr = indptr;
    fa.part_ptr = part_ptr;
    fa.part_row = g->part_row.as<int32_t>();
    fa.n_parts = g->c.n_parts;
    fa.part_edges = part_edges;
    fa.targets = targets;
    fa.qdeg = qdeg;
    fa.cand_row = cand_row;
    fa.node = ctx->node;
    fa.base_indptr = ctx->base.indptr;
    fa.base_indices = ctx->base.indices;
    fa.n_query = n_query;
    fa.raw_q = raw_q;
    fa.raw_t = raw_t;
    fa.cand_start = tcur;
    fa.target_slot = target_slot;
    fa.cols = cols;
    fa.cdeg = g->cdeg.as<int32_t>();
    fa.lg_group = 3;
    while (fa.lg_group < 6 && ((int64_t)g->c.n_parts << fa.lg_group) < g->c.nnz_in) ++fa.lg_group;
    // a request of a few thousand edges, built by one block: its second half is one block's work as well
    const bool tiny_tail = small && ctx->small_path != 2 && n_e > 0 && g->c.n_parts > 0 && g->c.n_parts <= 2048 && g->c.nnz_in <= 16384;
    {
        // A table larger than the memory-side cache whose rows this batch reads several times over: the inner
        // layers then walk their work items by table region (see k_phase_offsets); decided from the sizes the
        // caller announced for its largest such table.
        int32_t* order = nullptr;
        if (g->c.n_parts > 0 && !small && ctx->hint_table_bytes > OMG_ORDER_MIN_TABLE_BYTES &&
            omg_order_pays(g->c.nnz_in * ctx->hint_row_bytes, ctx->hint_table_bytes) &&
            g->c.n_parts < ((int64_t)1 << 31) && g->order.ensure(sizeof(int32_t) * (size_t)(g->c.n_parts + 1)) == OMG_OK) {
            order = g->order.as<int32_t>();
            g->order_ready = true;
        }
        SortFillArgs a{};
        a.nb_radix = sorts ? g->c.n_med + n_sub : 0;
        a.nb_wave = sorts && g->c.n_small > 0 ? (int64_t)grid_for(g->c.n_small, TPB / 64) : 0;
        a.list_med = list_med;
        a.list_small = list_small;
        a.n_med = g->c.n_med;
        a.n_small = g->c.n_small;
        a.n_sub = n_sub;
        a.n_query = n_query;
        a.indptr = indptr;
        a.qdeg = qdeg;
        a.target_slot = target_slot;
        a.bits_node = bn;
        a.bits_query = bq;
        a.sub = sub;
        a.raw = raw;
        a.cols = cols;
        a.part_ptr = part_ptr;
        a.rows_in = g->rows_in;
        a.n_parts = g->c.n_parts;
        a.part_row = g->part_row.as<int32_t>();
        a.phase_total = (const long long*)st->phase_total;
        a.phase_rank = st->phase_rank;
        a.order = order;
        const int64_t nb_fill = g->c.n_parts > 0 ? (int64_t)grid_for(g->c.n_parts) : 0;
        const int64_t nb = a.nb_radix + a.nb_wave + nb_fill;
        if (nb >= ((int64_t)1 << 31)) return OMG_ERANGE;
        if (tiny_tail) {
            // (the work list is written by k_finish_small below)
        } else if (nb > 0 && a.nb_radix > 0) {
            hipLaunchKernelGGL(k_sort_fill<true>, dim3((unsigned)nb), dim3(TPB), 0, s, a);
        } else if (nb > 0) {
            hipLaunchKernelGGL(k_sort_fill<false>, dim3((unsigned)nb), dim3(TPB), 0, s, a);
        }
    }
    if (tiny_tail) {
        hipLaunchKernelGGL(k_finish_small, dim3(1), dim3(1024), 0, s, fa, g->rows_in, (const int32_t*)cand, cd, max_cand,
                           ctx->node);
    } else {
        if (g->c.n_parts > 0 && n_e > 0)
            hipLaunchKernelGGL(k_finish_cols, dim3(grid_for(g->c.n_parts, TPB >> fa.lg_group)), dim3(TPB), 0, s, fa);
        if (n_e > 0) hipLaunchKernelGGL(k_clear_slots, dim3(gc), dim3(TPB), 0, s, cand, cd, max_cand, ctx->node);
    }
    ctx->slots_dirty = false;
    OMG_HIP(hipGetLastError());
    g->built = true;
    return OMG_OK;
}

// The node-to-slot map is -1 everywhere between builds.  A build that stops after the candidates were
// emitted (a rejected request, an allocation that failed once the sizes were known) has left this batch's
// slots in it; the next build would take those nodes for candidates.  Every such exit passes here.
int omg_build_impl(omg_ctx* ctx, omg_graph* g, int32_t n_query, int64_t n_e, const int32_t* qe_query,
                   const omg_node_t* qe_node, uint32_t gamma_ppm, const omg_node_t* rset, int64_t n_rset) {
    const int rc = build_body(ctx, g, n_query, n_e, qe_query, qe_node, gamma_ppm, rset, n_rset);
    if (rc != OMG_OK && ctx->slots_dirty) {
        const int64_t max_cand = n_e < ctx->base.n_nodes ? n_e : ctx->base.n_nodes;
        hipLaunchKernelGGL(k_clear_slots, dim3(grid_for(max_cand + 1)), dim3(TPB), 0, ctx->stream, g->cand.as<int32_t>(),
                           ctx->counts_dev, max_cand, ctx->node);
        (void)hipStreamSynchronize(ctx->stream);
        ctx->slots_dirty = false;
    }
    return rc;
}
