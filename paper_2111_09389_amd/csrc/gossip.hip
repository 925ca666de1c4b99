// Gossip step of Algorithm 1 (step 7) for n agents simulated on one GPU:
// plain neighbourhood averaging and CHOCO-SGD (supplement Algorithm 3) with
// exact layer-wise top-k of |x - xhat|.  Everything is HBM-bound streaming.
//
// Mixing: one thread owns one parameter column e and stages all n agents' values of
// it in its own LDS column, so the in-place update has no cross-thread hazard and
// each row is read once and written once.
//
// Top-k: MSB-first radix select on the 64-bit key (|v| bit pattern << 32 | ~index
// inside the segment).  Keys are unique, so "key >= k-th largest key" selects
// exactly k entries and resolves ties towards the lower index.  Pass 1 histograms
// the top 12 key bits over the full data; pass 2 copies the keys that fall in the
// threshold bin (a fraction of a percent of the data for smooth distributions) to
// a candidate list; the remaining 51 bits are resolved on the candidates only.
// Large problems take ONE pass over the full data instead: a histogram of a sample of
// the tiles guesses a window of bins around each threshold bin, the full pass counts
// the keys above the window and keeps the window's keys, and a pair whose window turns
// out to have missed the threshold bin is redone in the two-pass form (exact either way).
#include "common.h"
#include <cmath>
#include <atomic>
#include <cstdlib>
#include <cstring>
#include <type_traits>
#include <vector>

namespace lpdt {

constexpr int kMaxAgents = 64;
constexpr int kMaxDeg = 8;
constexpr int kGThreads = 256;
constexpr int kTile = 4096;        // elements per block in the full-data passes
constexpr int kBins = 4096;        // histogram bins per (agent, segment): the 12-bit first pass
constexpr int kUploadChunk = 384;  // int64 values per upload launch (kernel-argument space)

struct MixGraph {  // sparse rows of W, passed by value
    float w[kMaxAgents][kMaxDeg];
    uint8_t nbr[kMaxAgents][kMaxDeg];
    uint8_t deg[kMaxAgents];
};

// The same rows for graphs of at most 16 agents and 4 non-zeros per row (rings, tori), padded with zero weights on the
// agent itself: every row has exactly 4 terms, so the kernels' loops over agents and terms unroll completely and the
// compiler fetches the whole graph with a few scalar loads up front instead of a chain of dependent ones per term.
struct MixGraph4 {
    static constexpr int kFixedDeg = 4;
    float w[16][4];
    uint8_t nbr[16][4];
};
template <typename G> struct FixedDeg { static constexpr int value = 0; };
template <> struct FixedDeg<MixGraph4> { static constexpr int value = 4; };

struct UploadChunk { long long v[kUploadChunk]; };

struct PairState {        // one per (agent, segment)
    unsigned long long prefix;  // key bits fixed so far (right aligned); finally the threshold key
    unsigned int rank;          // the wanted key is the rank-th largest among keys matching prefix
    unsigned int cand;          // candidates stored
    unsigned int lo, hi;        // one-pass selection: the window of 12-bit bins whose keys the full pass keeps
    unsigned int redo;          // one-pass selection: the window missed the threshold bin, select this pair in two passes
    unsigned int above;         // one-pass selection: number of keys in bins above the window
};

// ---- plain mix ---------------------------------------------------------------
template <int NMAX, typename G>
__global__ __launch_bounds__(kGThreads) void mix_plain_kernel(float *__restrict__ x, int n, size_t d, G g, float rate,
                                                              const float *__restrict__ unew, float *__restrict__ z) {
    // column values staged in LDS: neighbour ids are run-time values, and LDS takes a
    // run-time row index where registers cannot.  Each thread touches its own column only.
    __shared__ float sv[NMAX][kGThreads];
    const size_t e = (size_t)blockIdx.x * kGThreads + threadIdx.x;
    if (e >= d) return;
    float v[NMAX];
#pragma unroll
    for (int i = 0; i < NMAX; ++i)  // all rows' loads in flight together
        if (i < n) v[i] = x[(size_t)i * d + e];
#pragma unroll
    for (int i = 0; i < NMAX; ++i)
        if (i < n) sv[i][threadIdx.x] = v[i];
    if constexpr (FixedDeg<G>::value > 0) {
#pragma unroll
        for (int i = 0; i < NMAX; ++i)
            if (i < n) {
                float s = 0.0f;
#pragma unroll
                for (int t = 0; t < FixedDeg<G>::value; ++t) s += g.w[i][t] * sv[g.nbr[i][t]][threadIdx.x];
                const float o = v[i] + rate * (s - v[i]);
                x[(size_t)i * d + e] = o;
                if (z) z[(size_t)i * d + e] = __fdiv_rn(o, unew[i]);
            }
    } else {
        for (int i = 0; i < n; ++i) {
            const float vi = sv[i][threadIdx.x];
            float s = 0.0f;
            for (int t = 0; t < g.deg[i]; ++t) s += g.w[i][t] * sv[g.nbr[i][t]][threadIdx.x];
            const float o = vi + rate * (s - vi);
            x[(size_t)i * d + e] = o;
            if (z) z[(size_t)i * d + e] = __fdiv_rn(o, unew[i]);
        }
    }
}

// ---- CHOCO: set-up -----------------------------------------------------------
__global__ void upload_kernel(UploadChunk c, long long *dst, int count) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) dst[i] = c.v[i];
}

__global__ void choco_init_kernel(PairState *st, const long long *kk, int n, int nseg, unsigned int *hist, size_t hist_words,
                                  unsigned int *any_redo) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < hist_words) hist[i] = 0u;
    if (i == 0) *any_redo = 0u;
    if (i < (size_t)n * nseg) {
        PairState s;
        s.prefix = 0ull;
        s.rank = (unsigned int)kk[i % nseg];
        s.cand = 0u;
        s.lo = 0u; s.hi = 0u; s.redo = 0u; s.above = 0u;
        st[i] = s;
    }
}

// The set-up in one launch when its three tables (segment offsets, per-segment k, sampled tiles) fit one kernel-argument
// chunk together: what three upload_kernel launches and choco_init_kernel do (four dependent launches of ~4 us each).
__global__ void choco_setup_kernel(UploadChunk c, int n_off, int n_k, int n_list, long long *d_off, long long *d_k, long long *d_list,
                                   PairState *st, int n, int nseg, unsigned int *hist, size_t hist_words, unsigned int *any_redo) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < (size_t)n_off) d_off[i] = c.v[i];
    if (i < (size_t)n_k) d_k[i] = c.v[n_off + i];
    if (i < (size_t)n_list) d_list[i] = c.v[n_off + n_k + i];
    if (i < hist_words) hist[i] = 0u;
    if (i == 0) *any_redo = 0u;
    if (i < (size_t)n * nseg) {
        PairState s;
        s.prefix = 0ull;
        s.rank = (unsigned int)c.v[n_off + i % nseg];
        s.cand = 0u;
        s.lo = 0u; s.hi = 0u; s.redo = 0u; s.above = 0u;
        st[i] = s;
    }
}

// The (non-empty) segment holding element e < off[nseg], found by the whole block at once: every thread tests the
// segments tid, tid + blockDim, ..., so the block waits for one round of loads instead of a binary search's chain.
// The caller's next __syncthreads() publishes *s_first.
__device__ __forceinline__ void find_segment_block(const long long *__restrict__ off, int nseg, long long e, int *s_first) {
    for (int s = threadIdx.x; s < nseg; s += blockDim.x)
        if (off[s] <= e && e < off[s + 1]) *s_first = s;
}

// what is compressed: x - xhat (CHOCO) or x + delta (Deep-Squeeze), one fp32 operation
__device__ __forceinline__ float compress_input(float xv, float sv, int ds) { return ds ? __fadd_rn(xv, sv) : __fsub_rn(xv, sv); }

__device__ __forceinline__ unsigned long long make_key(float xv, float hv, unsigned int idx_in_seg, int ds) {
    const float v = compress_input(xv, hv, ds);
    return ((unsigned long long)(__float_as_uint(v) & 0x7fffffffu) << 32) | (unsigned long long)(~idx_in_seg);
}

// Walks to the segment of element e; `end` caches off[s + 1] so the offsets are not re-read per element.
__device__ __forceinline__ void seek_segment(const long long *__restrict__ off, long long e, int &s, long long &end) {
    while (e >= end) { ++s; end = off[s + 1]; }
}

// Pass 1: histogram of key bits 62..51 (the top 12 bits of |v|).  VEC = 4: 16-byte loads (needs d % 4 == 0).
// Blocks walk over the tiles blockIdx.x, blockIdx.x + gridDim.x, ...; with a tile list (the sample of the one-pass
// selection) over the listed tiles instead.
// any_redo != NULL: only the pairs marked `redo` are counted (normally none: the block leaves at once).
template <int VEC>
__device__ __forceinline__ void hist_tile(long long tile, const float *__restrict__ x, const float *__restrict__ xhat, size_t d,
                                          const long long *__restrict__ off, int nseg, unsigned int *__restrict__ hist, int ds,
                                          const PairState *__restrict__ st, bool only_redo, unsigned int *sh, int *s_first,
                                          int *s_last, unsigned int *range) {
    const int agent = blockIdx.y;
    const long long e0 = tile * kTile;
    const long long e1 = min(e0 + (long long)kTile, (long long)d);
    for (int i = threadIdx.x; i < 4096; i += kGThreads) sh[i] = 0u;
    if (threadIdx.x == 0) { range[0] = 4095u; range[1] = 0u; }   // bins touched by a round: [min, max], two pairs in turn
    find_segment_block(off, nseg, e0, s_first);
    find_segment_block(off, nseg, e1 - 1, s_last);
    __syncthreads();
    const int sfirst = *s_first, slast = *s_last;
    const float *xr = x + (size_t)agent * d, *hr = xhat + (size_t)agent * d;
    unsigned int *gh_all = hist + (size_t)agent * nseg * kBins;
    // the thread's 16 elements (e0 + (it * kGThreads + tid) * VEC + u) as bin numbers, two per register
    constexpr int kIters = 16 / VEC;
    unsigned int bins[8];
#pragma unroll
    for (int it = 0; it < kIters; ++it) {
        const long long e = e0 + ((long long)it * kGThreads + threadIdx.x) * VEC;
        float xv[VEC], hv[VEC];
        if (VEC == 4) {
            float4 a = make_float4(0.f, 0.f, 0.f, 0.f), b = a;
            if (e < e1) { a = *reinterpret_cast<const float4 *>(xr + e); b = *reinterpret_cast<const float4 *>(hr + e); }
            xv[0] = a.x; xv[1] = a.y; xv[2] = a.z; xv[3] = a.w;
            hv[0] = b.x; hv[1] = b.y; hv[2] = b.z; hv[3] = b.w;
        } else {
            xv[0] = e < e1 ? xr[e] : 0.f; hv[0] = e < e1 ? hr[e] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < VEC; ++u) {
            const int j = it * VEC + u;
            const unsigned int bin = (__float_as_uint(compress_input(xv[u], hv[u], ds)) & 0x7fffffffu) >> 19;
            if (j % 2 == 0) bins[j / 2] = bin; else bins[j / 2] |= bin << 16;
        }
    }
    // One round per segment of the tile (almost always one): its elements into the LDS histogram, then the non-empty
    // bins into the pair's histogram, clearing the LDS copy for the next round.  No per-element global atomics.  Only
    // the range of bins the round touched is walked: a tile in a run of small tensors (a network's normalisation
    // parameters) has a dozen rounds, and walking all 4096 bins in each made those few tiles the whole launch's time.
    int round = 0;   // rounds done: they alternate between the two [min, max] pairs of `range`
    for (int sg = sfirst; sg <= slast; ++sg) {
        const long long lo = max(off[sg], e0), hi = min(off[sg + 1], e1);  // the segment's part of the tile
        if (lo >= hi) continue;                                            // (the same in every thread)
        if (only_redo && !st[(size_t)agent * nseg + sg].redo) continue;
        unsigned int *const rng = range + 2 * (round & 1), *const rng_next = range + 2 * (~round & 1);
        ++round;
        unsigned int bmin = 4095u, bmax = 0u;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const long long e = e0 + ((long long)(j / VEC) * kGThreads + threadIdx.x) * VEC + j % VEC;
            if (e >= lo && e < hi) {
                const unsigned int b = (bins[j / 2] >> (16 * (j % 2))) & 0xffffu;
                atomicAdd(&sh[b], 1u);
                bmin = min(bmin, b); bmax = max(bmax, b);
            }
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            bmin = min(bmin, (unsigned int)__shfl_xor((int)bmin, o, 64));
            bmax = max(bmax, (unsigned int)__shfl_xor((int)bmax, o, 64));
        }
        if (threadIdx.x % 64 == 0 && bmin <= bmax) { atomicMin(&rng[0], bmin); atomicMax(&rng[1], bmax); }
        __syncthreads();
        // the other pair was last read before the previous round's closing barrier and is next written after this
        // round's: now is the time to reset it
        if (threadIdx.x == 0) { rng_next[0] = 4095u; rng_next[1] = 0u; }
        unsigned int *gh = gh_all + (size_t)sg * kBins;
        const unsigned int r_lo = rng[0], r_hi = rng[1];   // nothing touched: 4095 > 0, nothing to walk
        for (unsigned int i = r_lo + threadIdx.x; i <= r_hi && r_lo <= r_hi; i += kGThreads) {
            const unsigned int c = sh[i];
            if (c) { atomicAdd(&gh[i], c); sh[i] = 0u; }
        }
        __syncthreads();
    }
}

template <int VEC>
__global__ __launch_bounds__(kGThreads) void choco_hist_kernel(const float *__restrict__ x, const float *__restrict__ xhat,
                                                               size_t d, const long long *__restrict__ off, int nseg,
                                                               unsigned int *__restrict__ hist, int ds,
                                                               const long long *__restrict__ tile_list, int ntiles,
                                                               const PairState *__restrict__ st,
                                                               const unsigned int *__restrict__ any_redo) {
    __shared__ unsigned int sh[4096];
    __shared__ unsigned int range[4];
    __shared__ int s_first, s_last;
    if (any_redo && *any_redo == 0u) return;
    for (int t = blockIdx.x; t < ntiles; t += gridDim.x) {
        hist_tile<VEC>(tile_list ? tile_list[t] : (long long)t, x, xhat, d, off, nseg, hist, ds, st, any_redo != nullptr, sh,
                       &s_first, &s_last, range);
        __syncthreads();
    }
}

// Finds, per (agent, segment), the bin holding the rank-th largest key; extends the
// prefix by `bits`, reduces the rank to the rank inside that bin, clears the histogram.
// mode 0: the histogram covers all keys matching the prefix.
// mode 1 (one-pass selection): it covers the bins of the guessed window [lo, hi] only and `above` counts the keys in
//   higher bins; a pair whose threshold bin is not in the window drops its candidates and is marked `redo`.
// mode 2: the marked pairs again, now with their full histogram; the others are left alone.
__global__ __launch_bounds__(kGThreads) void choco_scan_kernel(PairState *__restrict__ st, unsigned int *__restrict__ hist, int bits,
                                                               int mode, unsigned int *__restrict__ any_redo) {
    __shared__ unsigned int part[kGThreads];
    __shared__ unsigned int s_above;
    __shared__ int s_thread;
    const int pair = blockIdx.x;
    if (mode == 2 && (*any_redo == 0u || st[pair].redo == 0u)) return;
    unsigned int *h = hist + (size_t)pair * kBins;
    const int nb = 1 << bits, per = kBins / kGThreads;  // thread t owns bins [hi - per*t - per + 1, hi - per*t], descending
    const unsigned int rank = st[pair].rank;
    if (rank == 0u) {  // empty segment: nothing to select
        for (int i = threadIdx.x; i < kBins; i += kGThreads) h[i] = 0u;
        if (threadIdx.x == 0) st[pair].prefix = ~0ull;
        return;
    }
    // mode 1: only the window's bins were counted, the others are (still) zero and are neither read nor cleared
    const unsigned int lo = mode == 1 ? st[pair].lo : 0u, hi = mode == 1 ? st[pair].hi : (unsigned int)(kBins - 1);
    unsigned int mine[kBins / kGThreads];
    unsigned int sum = 0;
    for (int k = 0; k < per; ++k) {
        const int b = kBins - 1 - (threadIdx.x * per + k);
        mine[k] = (b < nb && (unsigned int)b >= lo && (unsigned int)b <= hi) ? h[b] : 0u;
        sum += mine[k];
    }
    part[threadIdx.x] = sum;
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned int run = mode == 1 ? st[pair].above : 0u;
        int t = kGThreads;  // stays there when the threshold bin is not among the counted ones (mode 1 only)
        if (run < rank)
            for (t = 0; t < kGThreads; ++t) {
                if (run + part[t] >= rank) break;
                run += part[t];
            }
        s_above = run;
        s_thread = t;
        if (t == kGThreads) {  // the window missed
            st[pair].cand = 0u;
            st[pair].redo = 1u;
            atomicOr(any_redo, 1u);
        }
    }
    __syncthreads();
    if ((int)threadIdx.x == s_thread) {
        unsigned int run = s_above;
        for (int k = 0; k < per; ++k) {
            if (run + mine[k] >= rank) {
                const int b = kBins - 1 - (threadIdx.x * per + k);
                st[pair].prefix = (st[pair].prefix << bits) | (unsigned long long)b;
                st[pair].rank = rank - run;
                break;
            }
            run += mine[k];
        }
    }
    for (unsigned int i = lo + threadIdx.x; i <= hi; i += kGThreads) h[i] = 0u;
}

// One-pass selection, step 1 of 2 (after a histogram of every stride-th tile): per (agent, segment), the window of bins
// that holds the threshold bin with near certainty.  With ns of the segment's len elements sampled, the wanted rank
// scales to r = rank * ns / len; the window spans the bins where the sample's count from the top reaches r - margin
// and r + margin, margin = 5 sqrt(r) + r / 16 + 4 (sampling noise is about sqrt(r); the rest covers tiles that differ).
// A fully sampled segment gets the exact bin, a segment without samples the whole range.  Clears the histogram.
__global__ __launch_bounds__(kGThreads) void choco_guess_kernel(PairState *__restrict__ st, unsigned int *__restrict__ hist,
                                                                const long long *__restrict__ off, int nseg) {
    __shared__ unsigned int part[kGThreads];
    __shared__ unsigned int s_lo, s_hi;
    const int pair = blockIdx.x, seg = pair % nseg;
    unsigned int *h = hist + (size_t)pair * kBins;
    constexpr int per = kBins / kGThreads;  // thread t owns bins kBins-1 - per*t - k, k = 0..per-1 (descending)
    unsigned int mine[per];
    unsigned int sum = 0;
    for (int k = 0; k < per; ++k) {
        const int b = kBins - 1 - (threadIdx.x * per + k);
        mine[k] = h[b];
        sum += mine[k];
        h[b] = 0u;
    }
    part[threadIdx.x] = sum;
    if (threadIdx.x == 0) { s_lo = 0u; s_hi = kBins - 1; }
    __syncthreads();
    unsigned int before = 0, ns = 0;
    for (int t = 0; t < kGThreads; ++t) {
        if (t < (int)threadIdx.x) before += part[t];
        ns += part[t];
    }
    const long long len = off[seg + 1] - off[seg];
    const unsigned int rank = st[pair].rank;
    if (ns == 0u || rank == 0u) {  // nothing sampled: keep every bin (small segments); empty segment: nothing to do
        if (threadIdx.x == 0) { st[pair].lo = 0u; st[pair].hi = kBins - 1; }
        return;
    }
    double r = (double)rank, margin = 0.0;
    if ((long long)ns < len) {
        r = (double)rank * (double)ns / (double)len;
        margin = 5.0 * sqrt(r) + r / 16.0 + 4.0;
    }
    const double top = r - margin < 1.0 ? 1.0 : floor(r - margin);  // count from the top at which the window opens
    const double bot = ceil(r + margin);                             // ... and closes (past the sample: down to bin 0)
    // the thread whose bins hold the top-th / bot-th largest sampled key writes that bin
    unsigned int run = before;
    for (int k = 0; k < per; ++k) {
        const unsigned int b = (unsigned int)(kBins - 1 - (threadIdx.x * per + k));
        const unsigned int next = run + mine[k];
        if ((double)run < top && top <= (double)next) s_hi = b;
        if ((double)run < bot && bot <= (double)next) s_lo = b;
        run = next;
    }
    __syncthreads();
    if (threadIdx.x == 0) { st[pair].lo = s_lo; st[pair].hi = s_hi; }
}

// One-pass selection, step 2 of 2: the only pass over all the data.  Per pair it counts the keys in bins above the window
// (`above`), histograms the window's bins and keeps the window's keys, which is all the scan needs to find the threshold
// bin inside the window and the refinement to finish there.  The bulk of the elements (below the window) cost a
// subtraction and two compares each: no atomics, so the pass runs at streaming speed.  A thread loads its 16 elements
// up front and notes the window's elements in a bit mask; each wave then reserves room in the pair's list for all its
// keys with one atomic and stores them from registers.  Elements of the tile that lie past its first segment (tiles
// with a segment boundary) are handled afterwards, one by one, with the windows of up to kSegCache following segments
// held in LDS.
constexpr int kSegCache = 32;
static_assert(kTile == kGThreads * 16, "one candidate bit per element of a thread: 16 elements per thread and tile");
template <int VEC>
__global__ __launch_bounds__(kGThreads) void choco_window_kernel(const float *__restrict__ x, const float *__restrict__ xhat,
                                                                 size_t d, const long long *__restrict__ off, int nseg,
                                                                 unsigned int *__restrict__ hist, PairState *__restrict__ st,
                                                                 unsigned long long *__restrict__ cand,
                                                                 unsigned int *__restrict__ tile_count, int ds) {
    __shared__ unsigned int sh[4096];
    __shared__ unsigned int wave_keys[kGThreads / kWave];
    __shared__ long long c_end[kSegCache];
    __shared__ unsigned int c_lo[kSegCache], c_hi[kSegCache], c_above[kSegCache];
    __shared__ int s_first, s_last;
    __shared__ unsigned int s_above;
    const int agent = blockIdx.y;
    const long long e0 = (long long)blockIdx.x * kTile;
    const long long e1 = min(e0 + (long long)kTile, (long long)d);
    constexpr int kIters = 16 / VEC;
    const float *xr = x + (size_t)agent * d, *hr = xhat + (size_t)agent * d;
    float xv[16], hv[16];  // element j = it * VEC + u of this thread: e0 + (it * kGThreads + threadIdx.x) * VEC + u
#pragma unroll
    for (int it = 0; it < kIters; ++it) {
        const long long e = e0 + ((long long)it * kGThreads + threadIdx.x) * VEC;
        if (VEC == 4) {
            float4 a = make_float4(0.f, 0.f, 0.f, 0.f), b = a;
            if (e < e1) {
                typedef float nt4 __attribute__((ext_vector_type(4)));
                const nt4 na = __builtin_nontemporal_load(reinterpret_cast<const nt4 *>(xr + e));
                const nt4 nb = __builtin_nontemporal_load(reinterpret_cast<const nt4 *>(hr + e));
                a = make_float4(na[0], na[1], na[2], na[3]); b = make_float4(nb[0], nb[1], nb[2], nb[3]);
            }
            xv[it * 4 + 0] = a.x; xv[it * 4 + 1] = a.y; xv[it * 4 + 2] = a.z; xv[it * 4 + 3] = a.w;
            hv[it * 4 + 0] = b.x; hv[it * 4 + 1] = b.y; hv[it * 4 + 2] = b.z; hv[it * 4 + 3] = b.w;
        } else {
            xv[it] = e < e1 ? xr[e] : 0.f;
            hv[it] = e < e1 ? hr[e] : 0.f;
        }
    }
    find_segment_block(off, nseg, e0, &s_first);
    find_segment_block(off, nseg, e1 - 1, &s_last);
    if (threadIdx.x == 0) s_above = 0u;
    __syncthreads();
    const int sfirst = s_first;
    const int nlater = s_last - sfirst;                       // segments of the tile after its first
    const int ncached = nlater < kSegCache ? nlater : kSegCache;
    PairState *pairs = st + (size_t)agent * nseg;
    if ((int)threadIdx.x < ncached) {
        const int sg = sfirst + 1 + threadIdx.x;
        c_end[threadIdx.x] = off[sg + 1];
        c_lo[threadIdx.x] = pairs[sg].lo;
        c_hi[threadIdx.x] = pairs[sg].hi;
        c_above[threadIdx.x] = 0u;
    }
    const long long first_begin = off[sfirst], first_end = off[sfirst + 1];
    PairState *pfirst = &pairs[sfirst];
    const unsigned int first_lo = pfirst->lo, first_hi = pfirst->hi, span = first_hi - first_lo;  // lo <= hi
    for (unsigned int i = first_lo + threadIdx.x; i <= first_hi; i += kGThreads) sh[i] = 0u;
    __syncthreads();
    unsigned int *gh_all = hist + (size_t)agent * nseg * kBins;
    unsigned long long *clist = cand + (size_t)agent * d;
    unsigned int marks = 0u, later = 0u, above = 0u;
#pragma unroll
    for (int j = 0; j < 16; ++j) {
        const long long e = e0 + ((long long)(j / VEC) * kGThreads + threadIdx.x) * VEC + j % VEC;
        if (e >= e1) continue;
        if (e >= first_end) { later |= 1u << j; continue; }
        const unsigned int bin = (__float_as_uint(compress_input(xv[j], hv[j], ds)) & 0x7fffffffu) >> 19;
        if (bin - first_lo <= span) {
            atomicAdd(&sh[bin], 1u);
            marks |= 1u << j;
        }
        above += bin > first_hi ? 1u : 0u;
    }
    // The keys of the tile's first segment go to the tile's own place in the pair's list, cand[e0 ...] (a tile has at
    // most as many keys as elements, so tiles never collide and nothing has to be reserved), packed: exclusive prefix
    // sum of the lanes' counts in the wave, then of the waves' totals.  tile_count tells the refinement how many.
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    const unsigned int mine = (unsigned int)__popc(marks);
    unsigned int incl = mine;
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        const unsigned int v = __shfl_up(incl, o, kWave);
        if (lane >= o) incl += v;
    }
    if (lane == kWave - 1) wave_keys[wave] = incl;
    __syncthreads();
    {
        unsigned int before = 0u, total = 0u;
#pragma unroll
        for (int w = 0; w < kGThreads / kWave; ++w) {
            if (w < wave) before += wave_keys[w];
            total += wave_keys[w];
        }
        if (threadIdx.x == 0) tile_count[(size_t)agent * gridDim.x + blockIdx.x] = total;
        unsigned long long *dst = clist + e0 + before + (incl - mine);
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            if (marks & (1u << j)) {
                const long long e = e0 + ((long long)(j / VEC) * kGThreads + threadIdx.x) * VEC + j % VEC;
                *dst++ = make_key(xv[j], hv[j], (unsigned int)(e - first_begin), ds);
            }
        }
    }
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) above += __shfl_xor(above, o, kWave);
    if (lane == 0 && above) atomicAdd(&s_above, above);
    // the tile's elements past its first segment (ascending e per thread, so the segment index only moves forward)
    if (later) {
        int k = 0;
        int sg = sfirst + 1 + ncached;     // for segments beyond the cached ones
        long long end_g = 0, begin_g = 0;
        bool walking = false;
        while (later) {
            const int j = __ffs(later) - 1;
            later &= later - 1u;
            const long long e = e0 + ((long long)(j / VEC) * kGThreads + threadIdx.x) * VEC + j % VEC;
            const float xe = xr[e], he = hr[e];
            const unsigned int bin = (__float_as_uint(compress_input(xe, he, ds)) & 0x7fffffffu) >> 19;
            while (k < ncached && e >= c_end[k]) ++k;
            if (k < ncached) {
                const long long begin = k ? c_end[k - 1] : first_end;
                const int sk = sfirst + 1 + k;
                if (bin > c_hi[k]) {
                    atomicAdd(&c_above[k], 1u);
                } else if (bin >= c_lo[k]) {
                    atomicAdd(&gh_all[(size_t)sk * kBins + bin], 1u);
                    clist[begin + atomicAdd(&pairs[sk].cand, 1u)] = make_key(xe, he, (unsigned int)(e - begin), ds);
                }
            } else {  // more segments in this tile than the cache holds: straight from memory
                if (!walking) { walking = true; begin_g = off[sg]; end_g = off[sg + 1]; }
                while (e >= end_g) { ++sg; begin_g = end_g; end_g = off[sg + 1]; }
                PairState *ps = &pairs[sg];
                if (bin > ps->hi) {
                    atomicAdd(&ps->above, 1u);
                } else if (bin >= ps->lo) {
                    atomicAdd(&gh_all[(size_t)sg * kBins + bin], 1u);
                    clist[begin_g + atomicAdd(&ps->cand, 1u)] = make_key(xe, he, (unsigned int)(e - begin_g), ds);
                }
            }
        }
    }
    __syncthreads();
    unsigned int *gh = gh_all + (size_t)sfirst * kBins;
    for (unsigned int i = first_lo + threadIdx.x; i <= first_hi; i += kGThreads)
        if (sh[i]) atomicAdd(&gh[i], sh[i]);
    if (threadIdx.x == 0 && s_above) atomicAdd(&pfirst->above, s_above);
    if ((int)threadIdx.x < ncached && c_above[threadIdx.x]) atomicAdd(&pairs[sfirst + 1 + threadIdx.x].above, c_above[threadIdx.x]);
}

// Pass 2: copy the keys whose top 12 bits equal the prefix to the candidate list of
// their (agent, segment); the list lives at the segment's own offset in `cand`.
// Matches of the block's first segment are gathered in LDS and get their room in the list
// with one global atomic per block; the (few) elements of later segments in the same tile
// reserve their slots one by one.
template <int VEC>
__device__ __forceinline__ void collect_tile(long long tile, const float *__restrict__ x, const float *__restrict__ xhat, size_t d,
                                             const long long *__restrict__ off, int nseg, PairState *__restrict__ st,
                                             unsigned long long *__restrict__ cand, int ds, bool only_redo,
                                             unsigned long long *stage, int *s_first, unsigned int *s_count, unsigned int *s_base) {
    const int agent = blockIdx.y;
    const long long e0 = tile * kTile;
    const long long e1 = min(e0 + (long long)kTile, (long long)d);
    find_segment_block(off, nseg, e0, s_first);
    if (threadIdx.x == 0) *s_count = 0u;
    __syncthreads();
    const int sfirst = *s_first;
    int s = sfirst;
    long long end = off[s + 1], begin = off[s];
    // a pair that is not to be collected gets a prefix no key has (keys >> 51 are below 2^12)
    const PairState first = st[(size_t)agent * nseg + sfirst];
    const unsigned long long first_prefix = (only_redo && !first.redo) ? ~0ull : first.prefix;
    const float *xr = x + (size_t)agent * d, *hr = xhat + (size_t)agent * d;
    for (long long e = e0 + (long long)threadIdx.x * VEC; e < e1; e += (long long)kGThreads * VEC) {
        float xv[VEC], hv[VEC];
        if (VEC == 4) {
            const float4 a = *reinterpret_cast<const float4 *>(xr + e), b = *reinterpret_cast<const float4 *>(hr + e);
            xv[0] = a.x; xv[1] = a.y; xv[2] = a.z; xv[3] = a.w;
            hv[0] = b.x; hv[1] = b.y; hv[2] = b.z; hv[3] = b.w;
        } else {
            xv[0] = xr[e]; hv[0] = hr[e];
        }
#pragma unroll
        for (int u = 0; u < VEC; ++u) {
            if (e + u >= end) { seek_segment(off, e + u, s, end); begin = off[s]; }
            const unsigned long long key = make_key(xv[u], hv[u], (unsigned int)(e + u - begin), ds);
            if (s == sfirst) {
                if ((key >> 51) == first_prefix) stage[atomicAdd(s_count, 1u)] = key;
            } else {
                PairState *ps = &st[(size_t)agent * nseg + s];
                if ((key >> 51) == ps->prefix && (!only_redo || ps->redo))
                    cand[(size_t)agent * d + begin + atomicAdd(&ps->cand, 1u)] = key;
            }
        }
    }
    __syncthreads();
    const unsigned int count = *s_count;
    if (count == 0u) return;
    if (threadIdx.x == 0) *s_base = atomicAdd(&st[(size_t)agent * nseg + sfirst].cand, count);
    __syncthreads();
    unsigned long long *dst = cand + (size_t)agent * d + off[sfirst] + *s_base;
    for (unsigned int i = threadIdx.x; i < count; i += kGThreads) dst[i] = stage[i];
}

// Blocks walk over the tiles blockIdx.x, blockIdx.x + gridDim.x, ...
// any_redo != NULL: the second collection of the one-pass selection, only for the pairs marked `redo` (normally none).
template <int VEC>
__global__ __launch_bounds__(kGThreads) void choco_collect_kernel(const float *__restrict__ x, const float *__restrict__ xhat,
                                                                  size_t d, const long long *__restrict__ off, int nseg,
                                                                  PairState *__restrict__ st,
                                                                  unsigned long long *__restrict__ cand, int ds, int ntiles,
                                                                  const unsigned int *__restrict__ any_redo) {
    __shared__ unsigned long long stage[kTile];
    __shared__ int s_first;
    __shared__ unsigned int s_count, s_base;
    if (any_redo && *any_redo == 0u) return;
    for (int t = blockIdx.x; t < ntiles; t += gridDim.x) {
        collect_tile<VEC>(t, x, xhat, d, off, nseg, st, cand, ds, any_redo != nullptr, stage, &s_first, &s_count, &s_base);
        __syncthreads();
    }
}

// Refinement: one block per (agent, segment) finishes the selection among the pair's candidates (the keys sharing the
// 12-bit prefix; a fraction of a per cent of the segment for bell-shaped data).  Four more radix rounds (13, 13, 13, 12
// bits) each histogram the keys that still match the prefix in LDS and pick the bin holding the wanted rank.  After
// the first round the survivors are normally a handful: they are copied to LDS and the remaining rounds never touch
// memory; if they do not fit (massive ties) the rounds keep streaming the candidate list.  On exit prefix = the full
// 63-bit key of the k-th largest element.
constexpr int kRefThreads = 1024;
constexpr int kRefList = 2048;

// Bin of the rank-th largest key in a histogram of nb bins (descending bin order), and how many keys lie above it.
__device__ __forceinline__ void select_bin(const unsigned int *hist, int nb, unsigned int rank, unsigned int *wave_tot,
                                           unsigned int *s_bin, unsigned int *s_above) {
    const int t = threadIdx.x, lane = t % 64, wave = t / 64;
    const int per = nb / kRefThreads;  // thread t owns bins nb-1 - t*per - k, k = 0..per-1
    unsigned int sum = 0;
    for (int k = 0; k < per; ++k) sum += hist[nb - 1 - (t * per + k)];
    unsigned int incl = sum;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const unsigned int v = __shfl_up(incl, o, 64);
        if (lane >= o) incl += v;
    }
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    unsigned int before = 0;
    for (int w = 0; w < wave; ++w) before += wave_tot[w];
    incl += before;
    const unsigned int excl = incl - sum;
    if (excl < rank && rank <= incl) {  // exactly one thread: the matching keys number at least rank
        unsigned int run = excl;
        for (int k = 0; k < per; ++k) {
            const int b = nb - 1 - (t * per + k);
            if (run + hist[b] >= rank) { *s_bin = (unsigned int)b; *s_above = run; break; }
            run += hist[b];
        }
    }
    __syncthreads();
}

// tile_count != NULL (one-pass selection): a pair's candidates are the list at its segment's offset (keys of the part of
// the segment that shares a tile with earlier segments; `cand` of them) plus, for every tile that starts inside the
// segment, tile_count keys at the tile's own offset.  A pair marked `redo` was collected again into the plain list.
__global__ __launch_bounds__(kRefThreads) void choco_refine_kernel(const unsigned long long *__restrict__ cand, size_t d,
                                                                   const long long *__restrict__ off, int nseg,
                                                                   PairState *__restrict__ st,
                                                                   const unsigned int *__restrict__ tile_count) {
    __shared__ unsigned int hist[8192];
    __shared__ unsigned long long list[kRefList];
    __shared__ unsigned int wave_tot[kRefThreads / 64];
    __shared__ unsigned int s_bin, s_above, s_cnt;
    const int pair = blockIdx.x, agent = pair / nseg, seg = pair % nseg;
    const PairState ps = st[pair];
    if (ps.rank == 0u) return;  // empty segment: the scan has set the prefix that selects nothing
    const long long begin = off[seg], end = off[seg + 1];
    const unsigned long long *ca = cand + (size_t)agent * d;
    const unsigned int count = ps.cand;
    const bool tiled = tile_count != nullptr && ps.redo == 0u;
    const long long t0 = (begin + kTile - 1) / kTile, t1 = (end + kTile - 1) / kTile;  // tiles starting in [begin, end)
    const unsigned int ntiles_all = (unsigned int)((d + kTile - 1) / kTile);
    const unsigned int *tc = tiled ? tile_count + (size_t)agent * ntiles_all : nullptr;
    auto for_each_candidate = [&](auto f) {
        for (unsigned int i = threadIdx.x; i < count; i += kRefThreads) f(ca[begin + i]);
        if (tiled) {
            // 64 threads share a tile (tiles hold some tens of keys for smooth data) and a wave has 4 tiles in flight:
            // their counts are fetched together, then their first keys
            constexpr long long kPerRound = (long long)(kRefThreads / 64) * 4;
            const int lane = threadIdx.x % 64, wave = threadIdx.x / 64;
            for (long long tb = t0 + wave * 4; tb < t1; tb += kPerRound) {
                unsigned int cnt[4];
                unsigned long long first[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) cnt[q] = tb + q < t1 ? tc[tb + q] : 0u;
#pragma unroll
                for (int q = 0; q < 4; ++q) first[q] = (unsigned int)lane < cnt[q] ? ca[(tb + q) * kTile + lane] : 0ull;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    if ((unsigned int)lane < cnt[q]) f(first[q]);
                    for (unsigned int slot = (unsigned int)lane + 64u; slot < cnt[q]; slot += 64u) f(ca[(tb + q) * kTile + slot]);
                }
            }
        }
    };
    if (count <= (unsigned int)kRefThreads && (!tiled || t0 >= t1)) {
        // A handful of candidates in one plain list (the small tensors: two thirds of a network's segments): one key per
        // thread, and the key with exactly rank - 1 matching keys above it is the answer (keys are unique: they carry
        // the element's index).  The four radix rounds below cost such a block 15 us, mostly barriers.
        const unsigned long long key = threadIdx.x < count ? ca[begin + threadIdx.x] : 0ull;
        const bool match = threadIdx.x < count && (key >> 51) == ps.prefix;
        list[threadIdx.x] = match ? key : 0ull;      // 0 is never counted as larger than anything
        __syncthreads();
        if (match) {
            unsigned int greater = 0;
            for (unsigned int j = 0; j < count; ++j) greater += list[j] > key ? 1u : 0u;
            if (greater + 1u == ps.rank) st[pair].prefix = key;
        }
        return;
    }
    unsigned long long prefix = ps.prefix;
    unsigned int rank = ps.rank, listed = 0;
    bool in_lds = false;
    const int shifts[4] = {38, 25, 12, 0}, widths[4] = {13, 13, 13, 12};
    for (int r = 0; r < 4; ++r) {
        const int shift = shifts[r], bits = widths[r], nb = 1 << bits;
        const unsigned long long mask = (unsigned long long)(nb - 1);
        for (int i = threadIdx.x; i < nb; i += kRefThreads) hist[i] = 0u;
        __syncthreads();
        if (in_lds) {
            for (unsigned int i = threadIdx.x; i < listed; i += kRefThreads) {
                const unsigned long long key = list[i];
                if ((key >> (shift + bits)) == prefix) atomicAdd(&hist[(key >> shift) & mask], 1u);
            }
        } else {
            for_each_candidate([&](unsigned long long key) {
                if ((key >> (shift + bits)) == prefix) atomicAdd(&hist[(key >> shift) & mask], 1u);
            });
        }
        __syncthreads();
        select_bin(hist, nb, rank, wave_tot, &s_bin, &s_above);
        prefix = (prefix << bits) | (unsigned long long)s_bin;
        rank -= s_above;
        if (r == 0 && hist[s_bin] <= (unsigned int)kRefList) {  // the same decision in every thread
            if (threadIdx.x == 0) s_cnt = 0u;
            __syncthreads();
            for_each_candidate([&](unsigned long long key) {
                if ((key >> shift) == prefix) list[atomicAdd(&s_cnt, 1u)] = key;
            });
            __syncthreads();
            listed = s_cnt;
            in_lds = true;
        }
        __syncthreads();  // everyone has read s_bin / hist before the next round clears them
    }
    if (threadIdx.x == 0) st[pair].prefix = prefix;
}

typedef float nt2 __attribute__((ext_vector_type(2)));   // the type of the streaming (nontemporal) 8-byte accesses

// Final pass: xhat += top-k(x - xhat) for every agent, then the gossip update of x.
// A thread owns VEC adjacent parameter columns (VEC * 4-byte loads per agent row).
template <int NMAX, int VEC, typename G>
__global__ __launch_bounds__(kGThreads) void choco_apply_mix_kernel(float *__restrict__ x, float *__restrict__ xhat, int n,
                                                                    size_t d, const long long *__restrict__ off, int nseg,
                                                                    const PairState *__restrict__ st, int select_all,
                                                                    G g, float rate, int ds, const float *__restrict__ unew,
                                                                    float *__restrict__ z) {
    __shared__ int s_first;
    __shared__ unsigned long long sprefix[NMAX];        // thresholds of the block's first segment
    __shared__ float sh[NMAX][VEC][kGThreads];          // this thread's columns of xhat (after the update)
    const long long e0 = (long long)blockIdx.x * kGThreads * VEC;
    find_segment_block(off, nseg, e0, &s_first);
    __syncthreads();
    const int sfirst = s_first;
    if ((int)threadIdx.x < n) sprefix[threadIdx.x] = select_all ? 0ull : st[(size_t)threadIdx.x * nseg + sfirst].prefix;
    __syncthreads();
    const long long e = e0 + (long long)threadIdx.x * VEC;
    if (e >= (long long)d) return;
    int seg[VEC];
    unsigned int idx[VEC];
    {
        int s = sfirst;
        long long end = off[s + 1], begin = off[s];
#pragma unroll
        for (int u = 0; u < VEC; ++u) {
            if (e + u >= end && e + u < (long long)d) { seek_segment(off, e + u, s, end); begin = off[s]; }
            seg[u] = s;
            idx[u] = (unsigned int)(e + u - begin);
        }
    }
    float xv[NMAX][VEC];
#pragma unroll
    for (int i = 0; i < NMAX; ++i)
        if (i < n) {
            float hv[VEC];
            if (VEC == 2) {
                const nt2 a = __builtin_nontemporal_load(reinterpret_cast<const nt2 *>(x + (size_t)i * d + e));
                const nt2 b = __builtin_nontemporal_load(reinterpret_cast<const nt2 *>(xhat + (size_t)i * d + e));
                xv[i][0] = a[0]; xv[i][VEC - 1] = a[1]; hv[0] = b[0]; hv[VEC - 1] = b[1];
            } else {
                xv[i][0] = x[(size_t)i * d + e]; hv[0] = xhat[(size_t)i * d + e];
            }
            bool any = false;
#pragma unroll
            for (int u = 0; u < VEC; ++u) {
                const unsigned long long key = make_key(xv[i][u], hv[u], idx[u], ds);
                const unsigned long long thr = seg[u] == sfirst ? sprefix[i] : (select_all ? 0ull : st[(size_t)i * nseg + seg[u]].prefix);
                const bool sel = key >= thr;
                if (ds) {  // Deep-Squeeze: sh = C[v] (what is sent), state = v - C[v] (what is kept back)
                    const float v = __fadd_rn(xv[i][u], hv[u]);
                    sh[i][u][threadIdx.x] = sel ? v : 0.0f;
                    hv[u] = sel ? __fsub_rn(v, v) : v;
                    any = true;
                } else {   // CHOCO: sh = state = xhat + TopK(x - xhat)
                    if (sel) { hv[u] = __fadd_rn(hv[u], __fsub_rn(xv[i][u], hv[u])); any = true; }
                    sh[i][u][threadIdx.x] = hv[u];
                }
            }
            if (any) {
                if (VEC == 2) *reinterpret_cast<float2 *>(xhat + (size_t)i * d + e) = make_float2(hv[0], hv[VEC - 1]);
                else xhat[(size_t)i * d + e] = hv[0];
            }
        }
    // Mixing.  CHOCO with a row-stochastic W: sum_j W_ij (xhat_j - xhat_i), as printed.  With push-sum weights the rows
    // of W need not sum to 1 and all variants mix by (W - I): sum_j W_ij m_j - m_i, written for CHOCO as the printed sum
    // plus (rowsum_i - 1) * xhat_i so that the small differences are still formed first.
    const bool push = unew != nullptr;
#pragma unroll
    for (int i = 0; i < NMAX; ++i)
        if (i < n) {
            float o[VEC];
#pragma unroll
            for (int u = 0; u < VEC; ++u) {
                const float hi = sh[i][u][threadIdx.x];
                const float ref = ds ? 0.0f : hi;
                float sum = 0.0f, rs = 0.0f;
                if constexpr (FixedDeg<G>::value > 0) {
#pragma unroll
                    for (int t = 0; t < FixedDeg<G>::value; ++t) {
                        sum += g.w[i][t] * (sh[g.nbr[i][t]][u][threadIdx.x] - ref);
                        rs += g.w[i][t];
                    }
                } else {
                    for (int t = 0; t < g.deg[i]; ++t) {
                        sum += g.w[i][t] * (sh[g.nbr[i][t]][u][threadIdx.x] - ref);
                        rs += g.w[i][t];
                    }
                }
                if (ds) sum -= hi;
                else if (push) sum += (rs - 1.0f) * hi;
                o[u] = xv[i][u] + rate * sum;
            }
            if (VEC == 2) __builtin_nontemporal_store(nt2{o[0], o[VEC - 1]}, reinterpret_cast<nt2 *>(x + (size_t)i * d + e));
            else x[(size_t)i * d + e] = o[0];
            if (z) {  // de-biased model z_i = x_i / u_i
                const float ui = unew[i];
                if (VEC == 2) *reinterpret_cast<float2 *>(z + (size_t)i * d + e) = make_float2(__fdiv_rn(o[0], ui), __fdiv_rn(o[VEC - 1], ui));
                else z[(size_t)i * d + e] = __fdiv_rn(o[0], ui);
            }
        }
}

// Push-sum bias weights: unew_i = u_i + rate * (sum_j W_ij u_j - u_i); a second launch copies them back once every
// reader of the old values is done.
template <typename G>
__global__ void pushsum_weights_kernel(const float *__restrict__ u, int n, G g, float rate, float *__restrict__ unew) {
    const int i = threadIdx.x;
    if (i >= n) return;
    float s = 0.0f;
    if constexpr (FixedDeg<G>::value > 0) {
        for (int t = 0; t < FixedDeg<G>::value; ++t) s += g.w[i][t] * u[g.nbr[i][t]];
    } else {
        for (int t = 0; t < g.deg[i]; ++t) s += g.w[i][t] * u[g.nbr[i][t]];
    }
    unew[i] = u[i] + rate * (s - u[i]);
}
__global__ void copy_small_kernel(const float *__restrict__ src, float *__restrict__ dst, int n) {
    if ((int)threadIdx.x < n) dst[threadIdx.x] = src[threadIdx.x];
}

struct ChocoLayout {
    size_t off_bytes, k_bytes, state_bytes, hist_bytes, cand_bytes, flag_bytes, tile_bytes, list_bytes, total;
};
static ChocoLayout choco_layout(int n, size_t d, int nseg) {
    ChocoLayout L;
    L.off_bytes = round_up((size_t)(nseg + 1) * sizeof(long long), 256);
    L.k_bytes = round_up((size_t)nseg * sizeof(long long), 256);
    L.state_bytes = round_up((size_t)n * nseg * sizeof(PairState), 256);
    L.hist_bytes = round_up((size_t)n * nseg * kBins * sizeof(unsigned int), 256);
    L.cand_bytes = round_up((size_t)n * d * sizeof(unsigned long long), 256);
    L.flag_bytes = 256;
    L.tile_bytes = round_up((size_t)n * ((d + kTile - 1) / kTile) * sizeof(unsigned int), 256);
    L.list_bytes = round_up(((d + kTile - 1) / kTile + 1) * sizeof(long long), 256);  // the sampled tiles
    L.total = L.off_bytes + L.k_bytes + L.state_bytes + L.hist_bytes + L.cand_bytes + L.flag_bytes + L.tile_bytes + L.list_bytes;
    return L;
}

static int build_graph(const float *W, int n, MixGraph *g, bool push_sum) {
    for (int i = 0; i < n; ++i) {
        int deg = 0;
        double row = 0.0;
        for (int j = 0; j < n; ++j) {
            const float w = W[(size_t)i * n + j];
            LPDT_REQUIRE(std::isfinite(w) && w >= 0.0f && w <= 1.0f, LPDT_EINVAL,
                         "gossip_mix: W[%d][%d] = %g is outside [0,1]", i, j, (double)w);
            row += w;
            if (w != 0.0f) {
                LPDT_REQUIRE(deg < kMaxDeg, LPDT_EUNSUPPORTED, "gossip_mix: row %d of W has more than %d non-zeros", i, kMaxDeg);
                g->w[i][deg] = w;
                g->nbr[i][deg] = (uint8_t)j;
                ++deg;
            }
        }
        LPDT_REQUIRE(push_sum || std::fabs(row - 1.0) <= 1e-5, LPDT_EINVAL, "gossip_mix: row %d of W sums to %.8f, not 1", i, row);
        g->deg[i] = (uint8_t)deg;
    }
    for (int j = 0; j < n; ++j) {
        double col = 0.0;
        for (int i = 0; i < n; ++i) col += W[(size_t)i * n + j];
        LPDT_REQUIRE(std::fabs(col - 1.0) <= 1e-5, LPDT_EINVAL,
                     "gossip_mix: column %d of W sums to %.8f, not 1 (W must be doubly stochastic; column stochastic with push-sum weights)", j, col);
    }
    return LPDT_OK;
}

// Fills the padded 4-term form; false when the graph does not fit it.
static bool compact_graph(const MixGraph &g, int n, MixGraph4 *c) {
    if (n > 16) return false;
    for (int i = 0; i < 16; ++i)
        for (int t = 0; t < 4; ++t) { c->w[i][t] = 0.0f; c->nbr[i][t] = (uint8_t)(i < n ? i : 0); }
    for (int i = 0; i < n; ++i) {
        if (g.deg[i] > 4) return false;
        for (int t = 0; t < g.deg[i]; ++t) { c->w[i][t] = g.w[i][t]; c->nbr[i][t] = g.nbr[i][t]; }
    }
    return true;
}

// Tile stride of the sample for the one-pass selection, or 0 for the two-pass form.  Below some tens of millions of
// elements the three extra (small) launches cost more than the saved pass.  lpdt_gossip_set_sample_stride overrides the
// choice (0: always two passes; s > 0: one pass with every s-th tile sampled, whatever the size): for tests and tuning.
static std::atomic<int> g_sample_stride{-1};
static int one_pass_stride(int n, size_t d) {
    const int v = g_sample_stride.load(std::memory_order_relaxed);
    if (v >= 0) return v > 4096 ? 4096 : v;
    return (size_t)n * d >= ((size_t)32 << 20) ? 16 : 0;
}

template <typename F>
static void dispatch_nmax(int n, F f) {
    if (n <= 8) f(std::integral_constant<int, 8>());
    else if (n <= 16) f(std::integral_constant<int, 16>());
    else if (n <= 32) f(std::integral_constant<int, 32>());
    else f(std::integral_constant<int, 64>());
}

static void upload(const long long *src, int count, long long *dst, hipStream_t st) {
    for (int o = 0; o < count; o += kUploadChunk) {
        UploadChunk c;
        const int m = count - o < kUploadChunk ? count - o : kUploadChunk;
        for (int i = 0; i < m; ++i) c.v[i] = src[o + i];
        hipLaunchKernelGGL(upload_kernel, dim3((m + 127) / 128), dim3(128), 0, st, c, dst + o, m);
    }
}

}  // namespace lpdt

using namespace lpdt;

static size_t mix_workspace(int n, size_t d, int nseg, bool compressed, bool push_sum) {
    if (n <= 0 || d == 0) return 0;
    if (nseg <= 0) nseg = 1;
    return (compressed ? choco_layout(n, d, nseg).total : 0) + (push_sum ? 256 : 0);
}

extern "C" size_t lpdt_gossip_mix_workspace_bytes(int n, size_t d, int nseg, int choco) {
    return mix_workspace(n, d, nseg, choco != 0, false);
}
extern "C" size_t lpdt_gossip_mix_ex_workspace_bytes(int n, size_t d, int nseg, int mode, int push_sum) {
    return mix_workspace(n, d, nseg, mode != LPDT_MIX_PLAIN, push_sum != 0);
}

// mode: LPDT_MIX_*; state: xhat (CHOCO) / delta (Deep-Squeeze); u, z: push-sum weights and de-biased models or NULL
static int mix_impl(float *x, float *state, int n, size_t d, const float *W, float rate, double keep_ratio,
                    const int64_t *seg_offsets, int nseg, int mode, float *u, float *z, void *ws, size_t ws_bytes, void *stream) {
    LPDT_REQUIRE(x && W, LPDT_EINVAL, "gossip_mix: x and W must be non-NULL");
    LPDT_REQUIRE(n > 0 && d > 0, LPDT_EINVAL, "gossip_mix: n and d must be positive");
    LPDT_REQUIRE(n <= kMaxAgents, LPDT_EUNSUPPORTED, "gossip_mix: at most %d agents", kMaxAgents);
    LPDT_REQUIRE(std::isfinite(rate), LPDT_EINVAL, "gossip_mix: rate must be finite");
    LPDT_REQUIRE((d + kGThreads - 1) / kGThreads <= 0x7fffffffull, LPDT_EUNSUPPORTED, "gossip_mix: d too large");
    LPDT_REQUIRE(mode == LPDT_MIX_PLAIN || mode == LPDT_MIX_CHOCO || mode == LPDT_MIX_DEEPSQUEEZE, LPDT_EINVAL,
                 "gossip_mix: unknown mode %d", mode);
    LPDT_REQUIRE((mode == LPDT_MIX_PLAIN) == (state == nullptr), LPDT_EINVAL,
                 "gossip_mix: a compressed mode needs its state matrix (xhat / delta), the plain mix takes none");
    LPDT_REQUIRE(!z || u, LPDT_EINVAL, "gossip_mix: z (de-biased models) needs the push-sum weights u");
    const bool push = u != nullptr, ds = mode == LPDT_MIX_DEEPSQUEEZE;
    MixGraph g;
    std::memset(&g, 0, sizeof(g));
    int rc = build_graph(W, n, &g, push);
    if (rc) return rc;
    hipStream_t st = as_stream(stream);
    const unsigned int col_blocks = (unsigned int)((d + kGThreads - 1) / kGThreads);
    MixGraph4 g4;
    const bool fixed4 = compact_graph(g, n, &g4);

    std::vector<long long> off, kk;
    bool select_all = true;
    if (state) {
        LPDT_REQUIRE(keep_ratio > 0.0 && std::isfinite(keep_ratio), LPDT_EINVAL, "gossip_mix: keep_ratio must be positive");
        if (!seg_offsets || nseg <= 0) {
            nseg = 1;
            off = {0, (long long)d};
        } else {
            off.assign(seg_offsets, seg_offsets + nseg + 1);
            LPDT_REQUIRE(off[0] == 0 && off[nseg] == (long long)d, LPDT_EINVAL,
                         "gossip_mix: seg_offsets must start at 0 and end at d");
        }
        for (int s = 0; s < nseg; ++s) {
            const long long len = off[s + 1] - off[s];
            LPDT_REQUIRE(len >= 0, LPDT_EINVAL, "gossip_mix: seg_offsets must be non-decreasing");
            LPDT_REQUIRE(len < 0x7fffffffLL, LPDT_EUNSUPPORTED, "gossip_mix: segment %d has 2^31-1 or more elements", s);
            long long k = (long long)std::ceil(keep_ratio * (double)len);
            if (k < 1) k = 1;
            if (k > len) k = len;
            if (k < len) select_all = false;
            kk.push_back(k);
        }
    }
    rc = check_ws(ws, ws_bytes, mix_workspace(n, d, nseg, state != nullptr, push));
    if (rc) return rc;
    char *base = static_cast<char *>(ws);
    float *unew = nullptr;
    if (push) {  // the last 256 bytes of the workspace
        unew = reinterpret_cast<float *>(base + mix_workspace(n, d, nseg, state != nullptr, false));
        if (fixed4) hipLaunchKernelGGL(pushsum_weights_kernel<MixGraph4>, dim3(1), dim3(64), 0, st, u, n, g4, rate, unew);
        else hipLaunchKernelGGL(pushsum_weights_kernel<MixGraph>, dim3(1), dim3(64), 0, st, u, n, g, rate, unew);
    }

    if (!state) {
        dispatch_nmax(n, [&](auto tag) {
            constexpr int NMAX = decltype(tag)::value;
            if (NMAX <= 16 && fixed4)
                hipLaunchKernelGGL((mix_plain_kernel<(NMAX <= 16 ? NMAX : 16), MixGraph4>), dim3(col_blocks), dim3(kGThreads), 0, st, x, n,
                                   d, g4, rate, unew, z);
            else
                hipLaunchKernelGGL((mix_plain_kernel<NMAX, MixGraph>), dim3(col_blocks), dim3(kGThreads), 0, st, x, n, d, g, rate, unew, z);
        });
    } else {
        const ChocoLayout L = choco_layout(n, d, nseg);
        long long *d_off = reinterpret_cast<long long *>(base);
        long long *d_k = reinterpret_cast<long long *>(base + L.off_bytes);
        PairState *d_st = reinterpret_cast<PairState *>(base + L.off_bytes + L.k_bytes);
        unsigned int *d_hist = reinterpret_cast<unsigned int *>(base + L.off_bytes + L.k_bytes + L.state_bytes);
        unsigned long long *d_cand =
            reinterpret_cast<unsigned long long *>(base + L.off_bytes + L.k_bytes + L.state_bytes + L.hist_bytes);
        float *xhat = state;
        const int dsi = ds ? 1 : 0;
        if (select_all) upload(off.data(), nseg + 1, d_off, st);
        if (!select_all) {
            const size_t hist_words = (size_t)n * nseg * kBins;
            unsigned int *d_redo = reinterpret_cast<unsigned int *>(base + L.off_bytes + L.k_bytes + L.state_bytes + L.hist_bytes + L.cand_bytes);
            unsigned int *d_tiles = d_redo + L.flag_bytes / sizeof(unsigned int);
            const unsigned int ntiles = (unsigned int)((d + kTile - 1) / kTile);
            const dim3 tiles(ntiles, n);
            const bool vec4 = d % 4 == 0 && aligned(x, 16) && aligned(xhat, 16);
            const int stride = one_pass_stride(n, d);
            const long long *no_list = nullptr;
            const unsigned int *none = nullptr;
            // The sample of the one-pass selection (see below): every stride-th tile, and every tile with a segment boundary
            // in it, so that short segments are sampled completely and each longer one at least in the tiles of its two ends.
            std::vector<long long> list;
            long long *d_list = reinterpret_cast<long long *>(reinterpret_cast<char *>(d_tiles) + L.tile_bytes);
            if (stride > 0) {
                std::vector<char> mark(ntiles, 0);
                for (unsigned int t = 0; t < ntiles; t += (unsigned int)stride) mark[t] = 1;
                for (int sg = 1; sg < nseg; ++sg)
                    if (off[sg] > 0 && off[sg] < (long long)d && off[sg] % kTile != 0) mark[(size_t)(off[sg] / kTile)] = 1;
                for (unsigned int t = 0; t < ntiles; ++t)
                    if (mark[t]) list.push_back((long long)t);
            }
            if ((size_t)(nseg + 1) + (size_t)nseg + list.size() <= (size_t)kUploadChunk) {
                UploadChunk c;
                for (int i = 0; i <= nseg; ++i) c.v[i] = off[i];
                for (int i = 0; i < nseg; ++i) c.v[nseg + 1 + i] = kk[i];
                for (size_t i = 0; i < list.size(); ++i) c.v[2 * nseg + 1 + i] = list[i];
                size_t threads = hist_words > (size_t)kUploadChunk ? hist_words : (size_t)kUploadChunk;
                if (threads < (size_t)n * nseg) threads = (size_t)n * nseg;
                hipLaunchKernelGGL(choco_setup_kernel, dim3((unsigned int)((threads + 255) / 256)), dim3(256), 0, st, c, nseg + 1, nseg,
                                   (int)list.size(), d_off, d_k, d_list, d_st, n, nseg, d_hist, hist_words, d_redo);
            } else {
                upload(off.data(), nseg + 1, d_off, st);
                upload(kk.data(), nseg, d_k, st);
                hipLaunchKernelGGL(choco_init_kernel, dim3((unsigned int)((hist_words + 255) / 256)), dim3(256), 0, st, d_st, d_k, n,
                                   nseg, d_hist, hist_words, d_redo);
                if (!list.empty()) upload(list.data(), (int)list.size(), d_list, st);
            }
            if (stride > 0) {
                // One pass over the data instead of two: a histogram of a sample of the tiles guesses, per pair, a window
                // of bins around the threshold bin; the full pass counts the keys above the window, histograms the
                // window and keeps its keys; the scan finds the threshold bin in the window.  A pair whose window
                // missed (tiles that differ a lot from the sampled ones) goes through the two-pass form afterwards:
                // three launches that end at once when there is none.  The result is exact either way.
                const dim3 sampled((unsigned int)list.size(), n), few(ntiles < 128u ? ntiles : 128u, n);
                const int nl = (int)list.size(), nt = (int)ntiles;
                const unsigned int *redo = d_redo;
                if (vec4) hipLaunchKernelGGL(choco_hist_kernel<4>, sampled, dim3(kGThreads), 0, st, x, xhat, d, d_off, nseg, d_hist, dsi, (const long long *)d_list, nl, d_st, none);
                else hipLaunchKernelGGL(choco_hist_kernel<1>, sampled, dim3(kGThreads), 0, st, x, xhat, d, d_off, nseg, d_hist, dsi, (const long long *)d_list, nl, d_st, none);
                hipLaunchKernelGGL(choco_guess_kernel, dim3(n * nseg), dim3(kGThreads), 0, st, d_st, d_hist, d_off, nseg);
                if (vec4) hipLaunchKernelGGL(choco_window_kernel<4>, tiles, dim3(kGThreads), 0, st, x, xhat, d, d_off, nseg, d_hist, d_st, d_cand, d_tiles, dsi);
                else hipLaunchKernelGGL(choco_window_kernel<1>, tiles, dim3(kGThreads), 0, st, x, xhat, d, d_off, nseg, d_hist, d_st, d_cand, d_tiles, dsi);
                hipLaunchKernelGGL(choco_scan_kernel, dim3(n * nseg), dim3(kGThreads), 0, st, d_st, d_hist, 12, 1, d_redo);
                if (vec4) hipLaunchKernelGGL(choco_hist_kernel<4>, few, dim3(kGThreads), 0, st, x, xhat, d, d_off, nseg, d_hist, dsi, no_list, nt, d_st, redo);
                else hipLaunchKernelGGL(choco_hist_kernel<1>, few, dim3(kGThreads), 0, st, x, xhat, d, d_off, nseg, d_hist, dsi, no_list, nt, d_st, redo);
                hipLaunchKernelGGL(choco_scan_kernel, dim3(n * nseg), dim3(kGThreads), 0, st, d_st, d_hist, 12, 2, d_redo);
                if (vec4) hipLaunchKernelGGL(choco_collect_kernel<4>, few, dim3(kGThreads), 0, st, x, xhat, d, d_off, nseg, d_st, d_cand, dsi, nt, redo);
                else hipLaunchKernelGGL(choco_collect_kernel<1>, few, dim3(kGThreads), 0, st, x, xhat, d, d_off, nseg, d_st, d_cand, dsi, nt, redo);
            } else {
                const int nt = (int)ntiles;
                if (vec4) hipLaunchKernelGGL(choco_hist_kernel<4>, tiles, dim3(kGThreads), 0, st, x, xhat, d, d_off, nseg, d_hist, dsi, no_list, nt, d_st, none);
                else hipLaunchKernelGGL(choco_hist_kernel<1>, tiles, dim3(kGThreads), 0, st, x, xhat, d, d_off, nseg, d_hist, dsi, no_list, nt, d_st, none);
                hipLaunchKernelGGL(choco_scan_kernel, dim3(n * nseg), dim3(kGThreads), 0, st, d_st, d_hist, 12, 0, d_redo);
                if (vec4) hipLaunchKernelGGL(choco_collect_kernel<4>, tiles, dim3(kGThreads), 0, st, x, xhat, d, d_off, nseg, d_st, d_cand, dsi, nt, none);
                else hipLaunchKernelGGL(choco_collect_kernel<1>, tiles, dim3(kGThreads), 0, st, x, xhat, d, d_off, nseg, d_st, d_cand, dsi, nt, none);
            }
            hipLaunchKernelGGL(choco_refine_kernel, dim3(n * nseg), dim3(kRefThreads), 0, st, d_cand, d, d_off, nseg, d_st,
                               stride > 0 ? (const unsigned int *)d_tiles : (const unsigned int *)nullptr);
        }
        const bool vec2 = n <= 16 && d % 2 == 0 && aligned(x, 8) && aligned(xhat, 8) && (!z || aligned(z, 8));
        dispatch_nmax(n, [&](auto tag) {
            constexpr int NMAX = decltype(tag)::value;
            constexpr int N16 = NMAX <= 16 ? NMAX : 16;
            const dim3 grid2((unsigned)((d / 2 + kGThreads - 1) / kGThreads));
            if (NMAX <= 16 && vec2 && fixed4)
                hipLaunchKernelGGL((choco_apply_mix_kernel<N16, 2, MixGraph4>), grid2, dim3(kGThreads), 0, st, x, xhat, n, d, d_off, nseg, d_st,
                                   select_all ? 1 : 0, g4, rate, dsi, unew, z);
            else if (NMAX <= 16 && vec2)
                hipLaunchKernelGGL((choco_apply_mix_kernel<N16, 2, MixGraph>), grid2, dim3(kGThreads), 0, st, x, xhat, n, d, d_off, nseg, d_st,
                                   select_all ? 1 : 0, g, rate, dsi, unew, z);
            else
                hipLaunchKernelGGL((choco_apply_mix_kernel<NMAX, 1, MixGraph>), dim3(col_blocks), dim3(kGThreads), 0, st, x, xhat, n, d, d_off,
                                   nseg, d_st, select_all ? 1 : 0, g, rate, dsi, unew, z);
        });
    }
    if (push) hipLaunchKernelGGL(copy_small_kernel, dim3(1), dim3(64), 0, st, unew, u, n);
    return launch_status("lpdt_gossip_mix");
}

extern "C" int lpdt_gossip_mix(float *x, float *xhat, int n, size_t d, const float *W, float rate, double keep_ratio,
                               const int64_t *seg_offsets, int nseg, void *ws, size_t ws_bytes, void *stream) {
    return mix_impl(x, xhat, n, d, W, rate, keep_ratio, seg_offsets, nseg, xhat ? LPDT_MIX_CHOCO : LPDT_MIX_PLAIN, nullptr, nullptr,
                    ws, ws_bytes, stream);
}

extern "C" int lpdt_gossip_mix_ex(float *x, float *state, int n, size_t d, const float *W, float rate, double keep_ratio,
                                  const int64_t *seg_offsets, int nseg, int mode, float *u, float *z, void *ws, size_t ws_bytes,
                                  void *stream) {
    return mix_impl(x, state, n, d, W, rate, keep_ratio, seg_offsets, nseg, mode, u, z, ws, ws_bytes, stream);
}

extern "C" int lpdt_gossip_set_sample_stride(int stride) {
    LPDT_REQUIRE(stride >= -1, LPDT_EINVAL, "gossip_set_sample_stride: stride must be -1 (automatic), 0 (two passes) or positive");
    lpdt::g_sample_stride.store(stride, std::memory_order_relaxed);
    return LPDT_OK;
}
