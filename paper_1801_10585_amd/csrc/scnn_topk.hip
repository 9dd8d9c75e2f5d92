// The attention step (Sec. 3.2; Algorithm 1 steps 13, 15-17): per (sample,
// output channel) keep the k strongest non-zero responses, then compact the
// surviving sites into sorted output rows.
//
// Selection = most-significant-digit radix select on an order-preserving 32-bit
// key of the score.  The first digit (11 bits) is histogrammed over the whole
// response matrix; the entries that fall into the bin holding the k-th
// strongest one -- a few percent -- are then copied, with their position in the
// column, to a side buffer, and the remaining digits (11 + 10 bits) are settled
// there by one workgroup per column.  That yields the exact k-th largest key
// tau, the number n_eq of entries equal to it and how many of those, q, still
// fit.  An entry survives iff  key > tau, or key == tau and it is among the q
// equal entries of lowest lin; candidate sites are stored in ascending lin, so
// "lowest lin" is "smallest position", and the q-th smallest position among the
// equal entries (a second, ascending radix select on the side buffer) is the
// cut.  The response matrix is read three times in all: histogram, collection,
// and the final mask + compaction + write.
#include "scnn_internal.h"

namespace scnn {

// ------------------------------------------------------------------ layout conversion (standalone entry)
// Sample ranges of a sorted row list: cand_start[b] = first row of sample b.
__global__ __launch_bounds__(256) void k_rows_sample_bounds(Geom g, const int32_t* __restrict__ coords,
                                                            long long rows, int* __restrict__ cand_start,
                                                            int* __restrict__ tile_start, Counters* ctr) {
    const int stride = 1 + g.ndim;
    for (int b = threadIdx.x; b <= g.batch; b += blockDim.x) {
        long long lo = 0, hi = rows;  // first row with sample index >= b
        while (lo < hi) {
            long long mid = (lo + hi) >> 1;
            if (coords[mid * stride] < b) lo = mid + 1; else hi = mid;
        }
        cand_start[b] = (int)lo;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int acc = 0;
        for (int b = 0; b < g.batch; ++b) {
            tile_start[b] = acc;
            acc += (cand_start[b + 1] - cand_start[b] + kTileRows - 1) / kTileRows;
        }
        tile_start[g.batch] = acc;
        ctr->n_tiles = acc;
        ctr->n_cand = rows;
    }
}

hipError_t launch_rows_sample_bounds(const Geom& g, const int32_t* coords, long long rows, int* cand_start,
                                     int* tile_start, Counters* ctr, hipStream_t s) {
    hipLaunchKernelGGL(k_rows_sample_bounds, dim3(1), dim3(256), 0, s, g, coords, rows, cand_start, tile_start,
                       ctr);
    return hipGetLastError();
}

// Site-major rows -> planar tiles, through LDS so that both sides coalesce.
__global__ __launch_bounds__(256) void k_rows_to_planar(Geom g, const int32_t* __restrict__ coords,
                                                        const float* __restrict__ feats, int channels,
                                                        const int* __restrict__ cand_start,
                                                        const int* __restrict__ tile_start,
                                                        const Counters* __restrict__ ctr,
                                                        unsigned* __restrict__ cand_lin, float* __restrict__ resp) {
    __shared__ float s_t[kTileRows][65];
    const int n_tiles = (int)ctr->n_tiles;
    const int stride = 1 + g.ndim;
    for (int tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const int b = sample_of_tile(tile_start, g.batch, tile);
        const int first = cand_start[b] + (tile - tile_start[b]) * kTileRows;
        int nrows = cand_start[b + 1] - first;
        if (nrows > kTileRows) nrows = kTileRows;
        if (threadIdx.x < nrows) {
            int bb, c0, c1, c2;
            load_site(g, coords + (size_t)(first + threadIdx.x) * stride, bb, c0, c1, c2);
            unsigned lin = 0;
            if (site_in_grid(g, bb, c0, c1, c2)) lin = (unsigned)lin_of(g, c0, c1, c2);
            cand_lin[first + threadIdx.x] = lin;
        }
        for (int cc = 0; cc < channels; cc += 64) {
            const int cw = (channels - cc) < 64 ? (channels - cc) : 64;
            __syncthreads();
            for (int i = threadIdx.x; i < kTileRows * 64; i += 256) {
                const int r = i >> 6, c = i & 63;
                float v = 0.0f;
                if (r < nrows && c < cw) v = feats[(size_t)(first + r) * channels + cc + c];
                s_t[r][c] = v;
            }
            __syncthreads();
            for (int i = threadIdx.x; i < kTileRows * 64; i += 256) {
                const int c = i >> 7, r = i & 127;
                if (c < cw) resp[((size_t)tile * channels + cc + c) * kTileRows + r] = s_t[r][c];
            }
        }
    }
}

hipError_t launch_rows_to_planar(const Geom& g, const int32_t* coords, const float* feats, int channels,
                                 const int* cand_start, const int* tile_start, const Counters* ctr,
                                 long long tiles_cap, unsigned* cand_lin, float* resp, hipStream_t s) {
    long long blocks = tiles_cap < 1 ? 1 : (tiles_cap > 4096 ? 4096 : tiles_cap);
    hipLaunchKernelGGL(k_rows_to_planar, dim3((unsigned)blocks), dim3(256), 0, s, g, coords, feats, channels,
                       cand_start, tile_start, ctr, cand_lin, resp);
    return hipGetLastError();
}

// ------------------------------------------------------------------ radix select
constexpr int kSideStage = 4096;  // side-buffer entries staged in LDS per workgroup before a flush

// Rank search in a 2048-bin histogram held in LDS.  descending: find the bin holding the kk-th entry counted from
// the top bin; else from the bottom bin.  Returns the bin and the number of entries strictly before it in that
// order.  1 <= kk <= total must hold.  Contains __syncthreads(); s_res is two shared words.
__device__ inline void block_pick(const unsigned* s_h, long long kk, bool descending, unsigned* s_wave, int* s_res,
                                  int& bin_out, unsigned& before_out) {
    // Works for any block size that is a multiple of 64 and at least 256: the first 256 threads search, every
    // thread passes the same barriers.
    const bool active = threadIdx.x < 256;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    unsigned local = 0;  // thread t owns bins [8t, 8t+8)
    if (active) {
#pragma unroll
        for (int i = 0; i < 8; ++i) local += s_h[threadIdx.x * 8 + i];
    }
    unsigned inc = local;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const unsigned t = __shfl_up(inc, d, 64);
        if (lane >= d) inc += t;
    }
    if (active && lane == 63) s_wave[wave] = inc;
    __syncthreads();
    if (active) {
        unsigned base = 0, total = 0;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const unsigned x = s_wave[w];
            if (w < wave) base += x;
            total += x;
        }
        const unsigned excl = base + inc - local;
        const unsigned before_threads = descending ? total - excl - local : excl;
        if ((long long)before_threads < kk && kk <= (long long)before_threads + (long long)local) {
            unsigned before = before_threads;
            int bin = descending ? threadIdx.x * 8 + 7 : threadIdx.x * 8;
            for (int i = 0; i < 7; ++i) {
                const unsigned c = s_h[bin];
                if (kk <= (long long)before + (long long)c) break;
                before += c;
                bin += descending ? -1 : 1;
            }
            s_res[0] = bin;
            s_res[1] = (int)before;
        }
    }
    __syncthreads();
    bin_out = s_res[0];
    before_out = (unsigned)s_res[1];
    __syncthreads();
}

// grid = (columns, slices).  Histogram of the top 11 key bits over the column's entries.
__global__ __launch_bounds__(256) void k_hist0(int mode, int channels, const int* __restrict__ tile_start,
                                               const float* __restrict__ resp, unsigned* __restrict__ hist,
                                               long long k, ColState* __restrict__ cols, Counters* ctr,
                                               unsigned long long side_cap) {
    constexpr int U = 4;  // tiles per wave and iteration
    __shared__ unsigned s_hist[kHistBins];
    __shared__ unsigned s_wave[4];
    __shared__ int s_res[2];
    const int col = blockIdx.x;
    const int b = col / channels, oc = col - b * channels;
    for (int i = threadIdx.x; i < kHistBins; i += 256) s_hist[i] = 0;
    __syncthreads();
    const int t0 = tile_start[b], t1 = tile_start[b + 1];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int tile0 = t0 + (blockIdx.y * 4 + wave) * U; tile0 < t1; tile0 += 4 * U * gridDim.y) {
        unsigned key[U][2];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int tile = tile0 + u;
            const float* seg = resp + ((size_t)(tile < t1 ? tile : t0) * channels + oc) * kTileRows;
            const unsigned k0 = score_key(seg[lane], mode), k1 = score_key(seg[64 + lane], mode);
            key[u][0] = tile < t1 ? k0 : 0u;
            key[u][1] = tile < t1 ? k1 : 0u;
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int h = 0; h < 2; ++h)
                if (key[u][h] != 0u) atomicAdd(&s_hist[key[u][h] >> 21], 1u);
    }
    __syncthreads();
    unsigned* gh = hist + (size_t)col * kHistBins;
    for (int i = threadIdx.x; i < kHistBins; i += 256) {
        const unsigned c = s_hist[i];
        if (c) atomicAdd(&gh[i], c);
    }
    // The block that finishes a column last goes on to pick the bin of the k-th strongest entry and a slice of the
    // side buffer for that bin.  (cols[col].pad counts the column's finished blocks until the state is written.)
    // The histogram is only ever touched by device-scope atomics, which are performed at the point of coherence;
    // the barrier waits for this block's to be acknowledged, so no cache flush (fence) is needed before the count.
    __syncthreads();
    if (threadIdx.x == 0) s_res[0] = (atomicAdd(&cols[col].pad, 1u) == gridDim.y - 1) ? 1 : 0;
    __syncthreads();
    if (!s_res[0]) return;
    unsigned* s_h = s_hist;
    unsigned local = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const unsigned c = __hip_atomic_load(&gh[threadIdx.x * 8 + i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_h[threadIdx.x * 8 + i] = c;
        local += c;
    }
    unsigned total;
    (void)block_exclusive_scan_256(local, s_wave, total);
    ColState st;
    st.prefix = 0; st.tau = 0; st.k_rem = k; st.n_eq = 0; st.q = 0; st.n_nz = total; st.done = 0; st.cut = 0xffffffffu;
    st.side_off = 0; st.side_fill = 0; st.pad = 0;
    if (k <= 0) {
        st.done = 1;
        st.tau = 0xffffffffu;  // no key is stronger: nothing survives
    } else if ((long long)total <= k) {
        st.done = 1;           // fewer entries than k: all survive (tau = 0, every non-zero key is above it)
    }
    if (st.done) {
        if (threadIdx.x == 0) cols[col] = st;
        return;
    }
    int bin;
    unsigned before;
    block_pick(s_h, k, true, s_wave, s_res, bin, before);
    if (threadIdx.x == 0) {
        st.prefix = (unsigned)bin;
        st.k_rem = k - (long long)before;
        st.n_eq = s_h[bin];  // for now: entries in the bin = entries the side buffer will hold
        const unsigned long long off = atomicAdd(&ctr->side_cursor, (unsigned long long)st.n_eq);
        if (off + st.n_eq > side_cap) {  // cannot happen with the documented workspace size
            atomicOr(&ctr->flags, SCNN_FLAG_CAND_OVERFLOW);
            st.done = 1;
            st.tau = 0xffffffffu;
        }
        st.side_off = off;
        cols[col] = st;
    }
}

// grid = (columns, slices).  Copy the entries of the threshold bin, with their position in the column, to the
// column's slice of the side buffer (order within the slice does not matter).  Every wave stages its hits in its
// own piece of LDS and flushes it on its own, so the loop has no workgroup barrier.
__global__ __launch_bounds__(256) void k_collect(int mode, int channels, const int* __restrict__ tile_start,
                                                 const float* __restrict__ resp, ColState* __restrict__ cols,
                                                 uint2* __restrict__ side) {
    constexpr int U = 4;                 // tile pairs per wave and iteration
    constexpr int WCAP = kSideStage / 4; // staged entries per wave
    __shared__ uint2 s_buf[kSideStage];
    const int col = blockIdx.x;
    const ColState st = cols[col];
    if (st.done) return;
    const int b = col / channels, oc = col - b * channels;
    const int t0 = tile_start[b], t1 = tile_start[b + 1];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const unsigned long long lt_mask = (1ull << lane) - 1ull;
    uint2* wbuf = s_buf + wave * WCAP;
    int fill = 0;  // wave-uniform
    auto flush = [&]() {
        unsigned base = 0;
        if (lane == 0) base = atomicAdd(&cols[col].side_fill, (unsigned)fill);
        base = __shfl(base, 0, 64);
        for (int i = lane; i < fill; i += 64) side[st.side_off + base + i] = wbuf[i];
        fill = 0;
    };
    // a wave takes whole tiles (two 64-row halves), tiles wave, wave + 4, ... of the slice
    for (int tile0 = t0 + (blockIdx.y * 4 + wave) * U; tile0 < t1; tile0 += 4 * U * gridDim.y) {
        unsigned key[U][2];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int tile = tile0 + u;
            const float* seg = resp + ((size_t)(tile < t1 ? tile : t0) * channels + oc) * kTileRows;
            const unsigned k0 = score_key(seg[lane], mode), k1 = score_key(seg[64 + lane], mode);
            key[u][0] = tile < t1 ? k0 : 0u;
            key[u][1] = tile < t1 ? k1 : 0u;
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const bool hit = key[u][h] != 0u && (key[u][h] >> 21) == st.prefix;
                const unsigned long long m = __ballot(hit);
                if (hit)
                    wbuf[fill + __popcll(m & lt_mask)] =
                        make_uint2(key[u][h], (unsigned)(tile0 + u - t0) * kTileRows + (unsigned)(h * 64 + lane));
                fill += __popcll(m);
            }
        if (fill > WCAP - U * 128) flush();
    }
    if (fill > 0) flush();
}

// One block per column: settle the remaining 21 key bits on the side buffer, then, if the equal entries do not all
// fit, the position below which they do.
constexpr int kSideThreads = 1024;

__global__ __launch_bounds__(kSideThreads) void k_side_select(ColState* __restrict__ cols,
                                                              const uint2* __restrict__ side) {
    __shared__ unsigned s_h[kHistBins];
    __shared__ unsigned s_wave[4];
    __shared__ int s_res[2];
    const int col = blockIdx.x;
    ColState st = cols[col];
    if (st.done) return;
    const uint2* e = side + st.side_off;
    const unsigned m = st.n_eq;
    auto clear = [&]() {
        for (int i = threadIdx.x; i < kHistBins; i += kSideThreads) s_h[i] = 0;
        __syncthreads();
    };
    // histogram of digit(entry) over the entries that pass(entry), loads issued eight at a time
    auto histogram = [&](auto pass, auto digit) {
        for (unsigned i0 = threadIdx.x; i0 < m; i0 += kSideThreads * 8) {
            uint2 x[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const unsigned i = i0 + (unsigned)kSideThreads * u;
                x[u] = i < m ? e[i] : make_uint2(0u, 0u);
            }
            // Data with long runs of equal scores (unit input values) sends most lanes of a wave to one bin, and LDS
            // serves the atomics of a wave on one word one after the other: the lanes that share the first active
            // lane's bin add once, through that lane; the others add on their own.
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const bool valid = i0 + (unsigned)kSideThreads * u < m && pass(x[u]);
                const unsigned bin = valid ? digit(x[u]) : 0u;
                const unsigned long long act = __ballot(valid);
                if (act == 0ull) continue;  // (uniform)
                const int first = __ffsll((long long)act) - 1;
                const unsigned b0 = __shfl(bin, first, 64);
                const unsigned long long same = __ballot(valid && bin == b0);
                if ((int)(threadIdx.x & 63) == first) atomicAdd(&s_h[b0], (unsigned)__popcll(same));
                else if (valid && bin != b0) atomicAdd(&s_h[bin], 1u);
            }
        }
        __syncthreads();
    };
    int bin;
    unsigned before;
    // key bits [20:10]
    clear();
    histogram([](uint2) { return true; }, [](uint2 x) { return (x.x >> 10) & 0x7ffu; });
    block_pick(s_h, st.k_rem, true, s_wave, s_res, bin, before);
    const unsigned prefix2 = (st.prefix << 11) | (unsigned)bin;
    const long long k_rem = st.k_rem - (long long)before;
    // key bits [9:0]
    clear();
    histogram([prefix2](uint2 x) { return (x.x >> 10) == prefix2; }, [](uint2 x) { return x.x & 0x3ffu; });
    block_pick(s_h, k_rem, true, s_wave, s_res, bin, before);
    const unsigned tau = (prefix2 << 10) | (unsigned)bin;
    const unsigned n_eq = s_h[bin];
    const unsigned q = (unsigned)(k_rem - (long long)before);  // 1 <= q <= n_eq
    __syncthreads();
    unsigned cut = 0xffffffffu;
    if (q < n_eq) {
        // q-th smallest position among the entries equal to tau: ascending radix select on the position
        unsigned pprefix = 0;
        long long rank = q;
        for (int pass = 0; pass < 3; ++pass) {
            const int shift = pass == 0 ? 21 : (pass == 1 ? 10 : 0), bits = pass == 2 ? 10 : 11;
            clear();
            histogram([=](uint2 x) { return x.x == tau && (pass == 0 || (x.y >> (shift + bits)) == pprefix); },
                      [=](uint2 x) { return (x.y >> shift) & ((1u << bits) - 1u); });
            block_pick(s_h, rank, false, s_wave, s_res, bin, before);
            pprefix = (pprefix << bits) | (unsigned)bin;
            rank -= (long long)before;
        }
        cut = pprefix;
    }
    if (threadIdx.x == 0) {
        st.tau = tau;
        st.n_eq = n_eq;
        st.q = q;
        st.cut = cut;
        cols[col] = st;
    }
}

// The whole selection of a column in one workgroup, for columns that fit its registers (grids of at most 32768
// sites per sample: the paper's networks from the second resolution level on).  The same digit passes as above,
// 11 + 11 + 10 key bits and, when the equal entries do not all fit, 11 + 4 position bits, over keys read once;
// no global histogram, no side buffer and one launch instead of three (what such a layer costs is launches).
constexpr int kSmallThreads = 1024;
constexpr int kSmallPerThread = 32;
constexpr long long kSmallColumn = (long long)kSmallThreads * kSmallPerThread;  // entries of a column at most

__global__ __launch_bounds__(kSmallThreads) void k_select_small(int mode, int channels,
                                                                const int* __restrict__ tile_start,
                                                                const float* __restrict__ resp, long long k,
                                                                ColState* __restrict__ cols) {
    __shared__ unsigned s_h[kHistBins];
    __shared__ unsigned s_wave[4];
    __shared__ int s_res[2];
    __shared__ unsigned s_total;
    const int col = blockIdx.x;
    const int b = col / channels, oc = col - b * channels;
    const int t0 = tile_start[b], t1 = tile_start[b + 1];
    const unsigned n = (unsigned)(t1 - t0) * kTileRows;  // positions of the column (<= kSmallColumn, see the launcher)
    if (threadIdx.x == 0) s_total = 0;
    // entry u of the thread sits at position u * 1024 + thread: a wave reads 64 consecutive rows of one tile
    unsigned key[kSmallPerThread];
    unsigned mine = 0;
#pragma unroll
    for (int u = 0; u < kSmallPerThread; ++u) {
        const unsigned i = (unsigned)u * kSmallThreads + threadIdx.x;
        key[u] = 0u;
        if (i < n)
            key[u] = score_key(resp[((size_t)(t0 + (int)(i >> 7)) * channels + oc) * kTileRows + (i & 127u)], mode);
        mine += key[u] != 0u ? 1u : 0u;
    }
    __syncthreads();
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) mine += __shfl_xor(mine, d, 64);
    if ((threadIdx.x & 63) == 0 && mine) atomicAdd(&s_total, mine);
    // histogram of digit(key, position) over the entries that pass(key, position)
    auto histogram = [&](auto pass, auto digit) {
        for (int i = threadIdx.x; i < kHistBins; i += kSmallThreads) s_h[i] = 0;
        __syncthreads();
#pragma unroll
        for (int u = 0; u < kSmallPerThread; ++u) {
            const unsigned i = (unsigned)u * kSmallThreads + threadIdx.x;
            if (key[u] != 0u && pass(key[u], i)) atomicAdd(&s_h[digit(key[u], i)], 1u);
        }
        __syncthreads();
    };
    histogram([](unsigned, unsigned) { return true; }, [](unsigned x, unsigned) { return x >> 21; });
    ColState st;
    st.prefix = 0; st.tau = 0; st.k_rem = k; st.n_eq = 0; st.q = 0; st.n_nz = s_total; st.done = 1; st.cut = 0xffffffffu;
    st.side_off = 0; st.side_fill = 0; st.pad = 0;
    if (k <= 0) st.tau = 0xffffffffu;  // no key is stronger: nothing survives
    if (k <= 0 || (long long)st.n_nz <= k) {  // or fewer entries than k: all survive (tau = 0)
        if (threadIdx.x == 0) cols[col] = st;
        return;
    }
    int bin;
    unsigned before;
    block_pick(s_h, k, true, s_wave, s_res, bin, before);  // key bits [31:21]
    const unsigned prefix1 = (unsigned)bin;
    long long k_rem = k - (long long)before;
    histogram([prefix1](unsigned x, unsigned) { return (x >> 21) == prefix1; },
              [](unsigned x, unsigned) { return (x >> 10) & 0x7ffu; });
    block_pick(s_h, k_rem, true, s_wave, s_res, bin, before);  // key bits [20:10]
    const unsigned prefix2 = (prefix1 << 11) | (unsigned)bin;
    k_rem -= (long long)before;
    histogram([prefix2](unsigned x, unsigned) { return (x >> 10) == prefix2; },
              [](unsigned x, unsigned) { return x & 0x3ffu; });
    block_pick(s_h, k_rem, true, s_wave, s_res, bin, before);  // key bits [9:0]
    const unsigned tau = (prefix2 << 10) | (unsigned)bin;
    const unsigned n_eq = s_h[bin];
    const unsigned q = (unsigned)(k_rem - (long long)before);  // 1 <= q <= n_eq
    __syncthreads();
    unsigned cut = 0xffffffffu;
    if (q < n_eq) {  // q-th smallest position among the entries equal to tau (positions have 15 bits)
        histogram([tau](unsigned x, unsigned) { return x == tau; }, [](unsigned, unsigned i) { return i >> 4; });
        block_pick(s_h, (long long)q, false, s_wave, s_res, bin, before);
        const unsigned phi = (unsigned)bin;
        const long long rank = (long long)q - (long long)before;
        histogram([tau, phi](unsigned x, unsigned i) { return x == tau && (i >> 4) == phi; },
                  [](unsigned, unsigned i) { return i & 15u; });
        block_pick(s_h, rank, false, s_wave, s_res, bin, before);
        cut = (phi << 4) | (unsigned)bin;
    }
    if (threadIdx.x == 0) {
        st.prefix = prefix2 >> 11;
        st.tau = tau;
        st.k_rem = k_rem;
        st.n_eq = n_eq;
        st.q = q;
        st.cut = cut;
        cols[col] = st;
    }
}

hipError_t launch_topk(const Geom& g, int channels, long long k, int mode, const int* tile_start,
                       const float* resp, ColState* cols, unsigned* hist, uint2* side, unsigned long long side_cap,
                       Counters* ctr, hipStream_t s) {
    const int ncols = g.batch * channels;
    if (ncols > 0 && (long long)((g.N + kTileRows - 1) / kTileRows) * kTileRows <= kSmallColumn) {
        hipLaunchKernelGGL(k_select_small, dim3(ncols), dim3(kSmallThreads), 0, s, mode, channels, tile_start, resp, k,
                           cols);
        return hipGetLastError();
    }
    int slices = 4096 / (ncols > 0 ? ncols : 1);  // (cfg 4, 256 columns: 16 slices; 8 or 32 were 6 % slower)
    if (slices < 1) slices = 1;
    if (slices > 64) slices = 64;
    hipLaunchKernelGGL(k_hist0, dim3(ncols, slices), dim3(256), 0, s, mode, channels, tile_start, resp, hist, k, cols,
                       ctr, side_cap);
    hipLaunchKernelGGL(k_collect, dim3(ncols, slices), dim3(256), 0, s, mode, channels, tile_start, resp, cols, side);
    hipLaunchKernelGGL(k_side_select, dim3(ncols), dim3(kSideThreads), 0, s, cols, side);
    return hipGetLastError();
}

// ------------------------------------------------------------------ keep mask, ReLU, compaction, write (one pass)
// Tiles are taken in ascending order through a ticket counter; the number of surviving rows before a tile comes
// from a decoupled look-back over per-tile status words {status, count}: a tile first publishes its own count,
// then walks back over its predecessors' words until it meets an inclusive prefix.  A predecessor always belongs
// to a workgroup that is already running (tickets are handed out in order), so the wait is short; it is bounded
// all the same, and a wait that runs out is reported in the status bits instead of hanging.
constexpr unsigned long long kStateAggregate = 1ull << 62, kStateInclusive = 2ull << 62, kStateValueMask = (1ull << 62) - 1;
constexpr int kLookbackSpinLimit = 1 << 22;

// Decoupled look-back, run by the first wave of the workgroup: publishes this tile's count, then inspects its
// predecessors, nearest first, kLookbackSlices * 64 of them per step.  The tiles in flight advance together, so the
// nearest tile whose inclusive sum is known usually lies about as far back as there are workgroups; reading that
// whole stretch with one batch of loads costs one memory round trip instead of one per 64 tiles.
// Returns the number of surviving rows before the tile (valid in every lane).
constexpr int kLookbackSlices = 6;
// (one thread) makes a tile's own count known to its successors
__device__ inline void publish_count(unsigned long long* tile_state, int tile, int count) {
    __hip_atomic_store(&tile_state[tile], (tile == 0 ? kStateInclusive : kStateAggregate) | (unsigned long long)count,
                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// (first wave; the tile's count has been published) sums the counts of all predecessors
__device__ inline long long lookback_published(unsigned long long* tile_state, int tile, int count, Counters* ctr) {
    const int lane = threadIdx.x & 63;
    if (tile == 0) return 0;
    long long base = 0;
    int hi = tile - 1;  // nearest predecessor not yet accounted for
    int spins = 0;
    while (hi >= 0) {
        unsigned long long w[kLookbackSlices];
#pragma unroll
        for (int u = 0; u < kLookbackSlices; ++u) {
            const int j = hi - u * 64 - lane;
            w[u] = kStateAggregate;  // positions past tile 0 count as empty aggregates
            if (j >= 0) w[u] = __hip_atomic_load(&tile_state[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        long long v = 0;
        int consumed = 0;
        bool done = false;
#pragma unroll
        for (int u = 0; u < kLookbackSlices; ++u) {
            const unsigned status = (unsigned)(w[u] >> 62);
            const unsigned long long empty = __ballot(status == 0), incl = __ballot(status == 2);
            // the usable prefix of the slice ends at the first inclusive word, or before the first empty one
            const int first_incl = incl ? __ffsll((long long)incl) - 1 : 64;
            const int first_empty = empty ? __ffsll((long long)empty) - 1 : 64;
            const int usable = first_incl < first_empty ? first_incl + 1 : first_empty;  // lanes [0, usable)
            if (lane < usable) v += (long long)(w[u] & kStateValueMask);
            consumed += usable;
            if (first_incl < first_empty) {
                done = true;  // reached an inclusive prefix
                break;
            }
            if (usable < 64) break;  // an unpublished tile: look again from there
        }
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
        base += v;
        if (done) break;
        hi -= consumed;
        if (consumed == 0) {
            if (++spins > kLookbackSpinLimit) {
                if (lane == 0) atomicOr(&ctr->flags, SCNN_FLAG_INTERNAL);
                break;
            }
            __builtin_amdgcn_s_sleep(1);
        }
    }
    if (lane == 0)
        __hip_atomic_store(&tile_state[tile], kStateInclusive | (unsigned long long)(base + count), __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
    return base;
}
__device__ inline long long lookback_wave(unsigned long long* tile_state, int tile, int count, Counters* ctr) {
    if ((threadIdx.x & 63) == 0) publish_count(tile_state, tile, count);
    return lookback_published(tile_state, tile, count, ctr);
}

// (one thread) The next `n` tiles of the compaction pass's queue.  Read-modify-writes of one address are served one
// at a time, about 13 ns each on this chip (a plain load of the counter is no cheaper), so a pass over a few
// thousand tiles can be bound by its tickets alone, and a thousand workgroups asking at once wait 13 us for theirs.
// Hence: several tiles per ticket in the narrow kernel, whose tiles are small, and no ticket that is known to come
// back empty: a launch with at least as many workgroups as tickets takes one ticket per workgroup (`once`), and a
// workgroup that has seen the queue empty does not ask again.
__device__ inline unsigned take_ticket(Counters* ctr, unsigned n) { return atomicAdd(&ctr->ticket, n); }

// The result counters, written by the last workgroup of the compaction pass to end (nnz_out may be null: a later
// kernel writes them).  aux = second counter: the candidate count (aux_is_cand) or a host-side number.
__device__ inline void finish_if_last(Counters* ctr, long long* nnz_out, long long aux_imm, int aux_is_cand,
                                      long long out_capacity) {
    if (!nnz_out) return;
    __syncthreads();  // (waits for the workgroup's counter updates, all device-scope atomics, to be acknowledged)
    if (threadIdx.x != 0) return;
    if (atomicAdd(&ctr->finished, 1u) != gridDim.x - 1) return;
    const long long rows = __hip_atomic_load(&ctr->n_rows, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    unsigned flags = __hip_atomic_load(&ctr->flags, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (rows > out_capacity) flags |= SCNN_FLAG_OUT_OVERFLOW;
    nnz_out[0] = rows;
    nnz_out[1] = aux_is_cand ? ctr->n_cand : aux_imm;
    nnz_out[2] = (long long)flags;
    nnz_out[3] = 0;
}

__global__ __launch_bounds__(256) void k_select_write(Geom g, int channels, int mode, int relu,
                                                      const int* __restrict__ cand_start,
                                                      const int* __restrict__ tile_start,
                                                      const unsigned* __restrict__ cand_lin,
                                                      const float* __restrict__ resp,
                                                      const ColState* __restrict__ cols,
                                                      unsigned long long* tile_state, Counters* ctr,
                                                      int32_t* __restrict__ out_coords, float* __restrict__ out_feats,
                                                      long long out_capacity, long long* __restrict__ nnz_out,
                                                      long long aux_imm, int aux_is_cand) {
    __shared__ unsigned s_tau[1024];
    __shared__ unsigned s_cut[1024];
    __shared__ unsigned s_flag[kTileRows];
    __shared__ int s_rank[kTileRows];
    __shared__ int s_wcount[2];
    __shared__ float s_v[kTileRows][65];
    __shared__ int s_ticket;
    __shared__ long long s_base;

    const int n_tiles = (int)ctr->n_tiles;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const unsigned long long lt_mask = (1ull << lane) - 1ull;
    const int n_chunks = (channels + 63) / 64;
    int cur_b = -1;

    for (;;) {
        __syncthreads();  // s_ticket and the tile buffers of the previous round are no longer read
        if (threadIdx.x == 0) s_ticket = (int)take_ticket(ctr, 1u);
        __syncthreads();
        const int tile = s_ticket;
        if (tile >= n_tiles) break;
        const int b = sample_of_tile(tile_start, g.batch, tile);
        const int first = cand_start[b] + (tile - tile_start[b]) * kTileRows;
        const unsigned pos0 = (unsigned)(tile - tile_start[b]) * kTileRows;  // position of row 0 in its column
        if (b != cur_b) {
            for (int c = threadIdx.x; c < channels; c += 256) {
                const ColState* st = cols + (size_t)b * channels + c;
                s_tau[c] = st->tau;
                s_cut[c] = st->cut;
            }
            cur_b = b;
        }
        if (threadIdx.x < kTileRows) s_flag[threadIdx.x] = 0;
        __syncthreads();

        // A wave handles channels wave, wave + 4, ... over the tile's 128 rows, four channels per step so that
        // eight loads are in flight.
        auto process = [&](int oc_first, int oc_end, bool stage, int cc) {
            for (int ob = oc_first + wave; ob < oc_end; ob += 16) {
                float v[4][2];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int oc = ob + 4 * j;
                    const float* seg = resp + ((size_t)tile * channels + (oc < oc_end ? oc : ob)) * kTileRows;
                    v[j][0] = seg[lane];
                    v[j][1] = seg[64 + lane];
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int oc = ob + 4 * j;
                    if (oc < oc_end) {
                        const unsigned tau = s_tau[oc], cut = s_cut[oc];
#pragma unroll
                        for (int half = 0; half < 2; ++half) {
                            const int r = half * 64 + lane;
                            const float x = v[j][half];
                            const unsigned key = score_key(x, mode);
                            bool keep = key > tau || (key == tau && key != 0u && pos0 + (unsigned)r <= cut);
                            if (relu) keep = keep && (x > 0.0f);
                            if (keep) s_flag[r] = 1u;
                            if (stage) s_v[r][oc - cc] = keep ? x : 0.0f;
                        }
                    }
                }
            }
        };
        process(0, channels, n_chunks == 1, 0);  // with several chunks the row flags need every channel first
        __syncthreads();
        if (threadIdx.x < kTileRows) {
            const unsigned long long m = __ballot(s_flag[threadIdx.x] != 0u);
            s_rank[threadIdx.x] = __popcll(m & lt_mask);
            if (lane == 0) s_wcount[wave] = __popcll(m);
        }
        __syncthreads();
        const int count = s_wcount[0] + s_wcount[1];
        if (wave == 0) {
            const long long base = lookback_wave(tile_state, tile, count, ctr);
            if (lane == 0) {
                if (tile == n_tiles - 1)
                    __hip_atomic_store(&ctr->n_rows, base + count, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                s_base = base;
            }
        }
        __syncthreads();
        const long long base = s_base;
        if (threadIdx.x < kTileRows && s_flag[threadIdx.x]) {
            const int rank = s_rank[threadIdx.x] + (wave ? s_wcount[0] : 0);
            s_rank[threadIdx.x] = rank;
            const long long orow = base + rank;
            if (orow < out_capacity) {
                int c0, c1, c2;
                site_of(g, cand_lin[first + threadIdx.x], c0, c1, c2);
                store_site(g, out_coords + orow * (1 + g.ndim), b, c0, c1, c2);
            }
        }
        __syncthreads();
        for (int cc = 0; cc < channels; cc += 64) {
            const int cw = (channels - cc) < 64 ? (channels - cc) : 64;
            if (n_chunks > 1) {
                process(cc, cc + cw, true, cc);
                __syncthreads();
            }
            for (int i = threadIdx.x; i < kTileRows * 64; i += 256) {
                const int r = i >> 6, c = i & 63;
                if (c < cw && s_flag[r]) {
                    const long long orow = base + s_rank[r];
                    if (orow < out_capacity) out_feats[orow * channels + cc + c] = s_v[r][c];
                }
            }
            __syncthreads();
        }
    }
    finish_if_last(ctr, nnz_out, aux_imm, aux_is_cand, out_capacity);
}

// The same pass for up to 64 channels, software-pipelined over three tiles.  A workgroup holds tile X (being
// written), tile Y (loaded) and tile Z (its loads in flight).  Per step it decides which entries of Y survive and
// publishes Y's row count, takes the ticket for Z and issues Z's loads, and only then looks back for X and writes
// it.  A tile's count is therefore known to its successors a whole step before its own look-back, so that a
// look-back rarely finds a predecessor unpublished, and the reads of one tile overlap the writes of another.
// The rows of a tile that keep an entry are two 64-bit masks (rows 0..63, 64..127) in one of three rotating slots;
// a row's rank is a popcount.  Three barriers per step.
__global__ __launch_bounds__(256, 4) void k_select_write64(Geom g, int channels, int mode, int relu,
                                                        const int* __restrict__ cand_start,
                                                        const int* __restrict__ tile_start,
                                                        const unsigned* __restrict__ cand_lin,
                                                        const float* __restrict__ resp,
                                                        const ColState* __restrict__ cols,
                                                        unsigned long long* tile_state, Counters* ctr,
                                                        int32_t* __restrict__ out_coords,
                                                        float* __restrict__ out_feats, long long out_capacity,
                                                        long long* __restrict__ nnz_out, long long aux_imm,
                                                        int aux_is_cand) {
    __shared__ uint4 s_thr[64];  // per channel: {threshold if the position passes the cut, threshold if not, cut, -}
    __shared__ unsigned long long s_mask[3][2];
    __shared__ int s_rank[kTileRows];  // output row of a kept row of the tile being written, relative; -1 = dropped
    __shared__ float s_v[kTileRows][65];
    __shared__ int s_ticket;
    __shared__ long long s_base;

    const int n_tiles = (int)ctr->n_tiles;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const bool vec4 = (channels & 3) == 0 && ((size_t)out_feats & 15) == 0;  // rows are 16-byte aligned
    int cur_b = -1;

    // values of channel wave + 4*m at rows lane and lane + 64
    auto load_tile = [&](int tile, float (&v)[16][2]) {
        const float* seg = resp + ((size_t)tile * channels + wave) * kTileRows + lane;
#pragma unroll
        for (int m = 0; m < 16; ++m) {
            if (wave + 4 * m < channels) {  // (uniform in the wave)
                v[m][0] = seg[m * 4 * kTileRows];
                v[m][1] = seg[m * 4 * kTileRows + 64];
            }
        }
    };
    // Zeroes, in the registers, the thread's values that do not survive; the rows that keep an entry are OR-ed into
    // the slot's masks (the slot is zero on entry).  An entry survives iff its key exceeds a threshold that depends
    // on its position only through the tie cut: key > tau, or key >= tau (tau > 0) where the position is within
    // the cut -- the same rule as "above tau, or equal to tau, non-zero and not past the cut".
    auto decide = [&](int tile, int slot, float (&v)[16][2]) {
        const int b = sample_of_tile(tile_start, g.batch, tile);
        const unsigned pos0 = (unsigned)(tile - tile_start[b]) * kTileRows;  // position of row 0 in its column
        if (b != cur_b) {  // (uniform: every thread sees the same tiles; the thresholds' readers are past a barrier)
            if (threadIdx.x < channels) {
                const ColState* st = cols + (size_t)b * channels + threadIdx.x;
                const unsigned tau = st->tau;
                s_thr[threadIdx.x] = make_uint4(tau - (tau != 0u ? 1u : 0u), tau, st->cut, 0u);
            }
            cur_b = b;
            __syncthreads();
        }
        bool row0 = false, row1 = false;
        const unsigned p0 = pos0 + (unsigned)lane, p1 = p0 + 64u;
#pragma unroll
        for (int m = 0; m < 16; ++m) {
            const int oc = wave + 4 * m;
            if (oc < channels) {
                const uint4 t = s_thr[oc];
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    const float x = v[m][half];
                    const unsigned key = score_key(x, mode);
                    bool keep = key > ((half ? p1 : p0) <= t.z ? t.x : t.y);
                    if (relu) keep = keep && (x > 0.0f);
                    v[m][half] = keep ? x : 0.0f;
                    if (half == 0) row0 |= keep; else row1 |= keep;
                }
            }
        }
        const unsigned long long b0 = __ballot(row0), b1 = __ballot(row1);
        if (lane == 0) {
            if (b0) atomicOr(&s_mask[slot][0], b0);
            if (b1) atomicOr(&s_mask[slot][1], b1);
        }
    };
    // the surviving values of a tile (the others are zero already), from registers to the transposition buffer
    auto stage_tile = [&](const float (&v)[16][2]) {
#pragma unroll
        for (int m = 0; m < 16; ++m) {
            const int oc = wave + 4 * m;
            if (oc < channels) {
                s_v[lane][oc] = v[m][0];
                s_v[64 + lane][oc] = v[m][1];
            }
        }
    };
    // ranks of the rows of the tile about to be written (threads 0..127, between the step's last two barriers)
    auto rank_rows = [&](int slot) {
        if (threadIdx.x < kTileRows) {
            const unsigned long long m0 = s_mask[slot][0], m1 = s_mask[slot][1];
            const unsigned long long mine = wave ? m1 : m0, below = (1ull << lane) - 1ull;
            const int rank = (wave ? __popcll(m0) : 0) + __popcll(mine & below);
            s_rank[threadIdx.x] = ((mine >> lane) & 1ull) ? rank : -1;
        }
    };
    // write of the staged tile: rows before the tile in s_base, rows within it in s_rank
    auto write_tile = [&](int tile) {
        const int b = sample_of_tile(tile_start, g.batch, tile);
        const int first = cand_start[b] + (tile - tile_start[b]) * kTileRows;
        const long long base = s_base;
        if (threadIdx.x < kTileRows) {
            const int rank = s_rank[threadIdx.x];
            if (rank >= 0 && base + rank < out_capacity) {
                int c0, c1, c2;
                site_of(g, cand_lin[first + threadIdx.x], c0, c1, c2);
                store_site(g, out_coords + (base + rank) * (1 + g.ndim), b, c0, c1, c2);
            }
        }
        if (vec4) {  // 16 bytes per thread: 16 threads cover a row of 64 channels
            const int c = (threadIdx.x & 15) * 4;
            if (c < channels) {
#pragma unroll
                for (int it = 0; it < kTileRows / 16; ++it) {
                    const int r = (threadIdx.x >> 4) + 16 * it;
                    const int rank = s_rank[r];
                    if (rank >= 0 && base + rank < out_capacity) {
                        float4 q;
                        q.x = s_v[r][c];
                        q.y = s_v[r][c + 1];
                        q.z = s_v[r][c + 2];
                        q.w = s_v[r][c + 3];
                        *(float4*)(out_feats + (base + rank) * channels + c) = q;
                    }
                }
            }
        } else {
            for (int i = threadIdx.x; i < kTileRows * 64; i += 256) {
                const int r = i >> 6, c = i & 63;
                const int rank = s_rank[r];
                if (c < channels && rank >= 0 && base + rank < out_capacity)
                    out_feats[(base + rank) * channels + c] = s_v[r][c];
            }
        }
    };

    // (thread 0) the next tile of this workgroup; a launch with a workgroup per tile asks once
    const bool once = (long long)gridDim.x >= n_tiles;
    bool asked = false;
    auto next_tile = [&]() -> int {
        const int t = (once && asked) ? n_tiles : (int)take_ticket(ctr, 1u);
        asked = true;
        return t;  // (at or past n_tiles: no tile)
    };
    if (threadIdx.x < 6) s_mask[threadIdx.x >> 1][threadIdx.x & 1] = 0ull;
    if (threadIdx.x == 0) s_ticket = next_tile();
    __syncthreads();
    float va[16][2], vb[16][2];
    // prologue: X = first ticket (loaded, decided), Y = second ticket (loads in flight)
    int tile_x = s_ticket;
    if (tile_x >= n_tiles) {
        finish_if_last(ctr, nnz_out, aux_imm, aux_is_cand, out_capacity);
        return;
    }
    load_tile(tile_x, va);
    __syncthreads();  // (the ticket has been read)
    if (threadIdx.x == 0) s_ticket = next_tile();
    decide(tile_x, 0, va);
    __syncthreads();
    int tile_y = s_ticket;
    if (tile_y < n_tiles) load_tile(tile_y, vb);
    if (threadIdx.x == 0) publish_count(tile_state, tile_x, __popcll(s_mask[0][0]) + __popcll(s_mask[0][1]));
    int slot_x = 0, slot_y = 1, slot_z = 2;
    // One step: (P, Q) hold (X, Y).  Decide Y, move X to LDS, fetch Z into P's registers, write X.
    auto step = [&](float (&P)[16][2], float (&Q)[16][2]) {
        __syncthreads();  // the previous step's writes are done: s_v, s_base, s_rank, s_ticket and slot_z are free
        if (threadIdx.x == 0) s_ticket = tile_y < n_tiles ? next_tile() : n_tiles;
        if (tile_y < n_tiles) decide(tile_y, slot_y, Q);
        stage_tile(P);
        __syncthreads();  // Y's masks, the ticket and the staged tile are in place
        const int tile_z = s_ticket;
        if (tile_z < n_tiles) load_tile(tile_z, P);  // in flight during the look-back and the writes
        rank_rows(slot_x);
        if (wave == 0) {
            if (lane == 0) {
                s_mask[slot_z][0] = 0ull;  // (last read before this step's first barrier, next used after its last)
                s_mask[slot_z][1] = 0ull;
                if (tile_y < n_tiles)
                    publish_count(tile_state, tile_y, __popcll(s_mask[slot_y][0]) + __popcll(s_mask[slot_y][1]));
            }
            const int count = __popcll(s_mask[slot_x][0]) + __popcll(s_mask[slot_x][1]);
            const long long base = lookback_published(tile_state, tile_x, count, ctr);
            if (lane == 0) {
                if (tile_x == n_tiles - 1)
                    __hip_atomic_store(&ctr->n_rows, base + count, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                s_base = base;
            }
        }
        __syncthreads();  // s_base, s_rank
        write_tile(tile_x);
        tile_x = tile_y;
        tile_y = tile_z;
        const int t = slot_x;
        slot_x = slot_y;
        slot_y = slot_z;
        slot_z = t;
    };
    for (;;) {
        step(va, vb);
        if (tile_x >= n_tiles) break;
        step(vb, va);
        if (tile_x >= n_tiles) break;
    }
    finish_if_last(ctr, nnz_out, aux_imm, aux_is_cand, out_capacity);
}

__global__ void k_finish(const Counters* __restrict__ ctr, int which_rows, long long aux_imm, int aux_is_cand,
                         long long out_capacity, long long* __restrict__ nnz_out) {
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        const long long rows = which_rows ? ctr->n_pool : ctr->n_rows;
        unsigned flags = ctr->flags;
        if (rows > out_capacity) flags |= SCNN_FLAG_OUT_OVERFLOW;
        nnz_out[0] = rows;
        nnz_out[1] = aux_is_cand ? ctr->n_cand : aux_imm;
        nnz_out[2] = (long long)flags;
        nnz_out[3] = 0;
    }
}

hipError_t launch_finish(const Counters* ctr, int which_rows, long long aux_imm, int aux_is_cand,
                         long long out_capacity, long long* nnz_out, hipStream_t s) {
    hipLaunchKernelGGL(k_finish, dim3(1), dim3(64), 0, s, ctr, which_rows, aux_imm, aux_is_cand, out_capacity,
                       nnz_out);
    return hipGetLastError();
}

// The same pass for narrow layers (at most 16 channels, the widths of the paper's own networks): a tile of 128 rows
// holds too little data to pay for a ticket, a look-back and three barriers, so a workgroup takes kNarrowTiles
// consecutive tiles per ticket (a "super-tile", one status word in tile_state) and a thread owns whole rows: it reads
// a row's channels from the planar tile (coalesced across the wave), decides them, and writes the row itself.
template <int CMAX, int kNarrowTiles /* tiles per ticket at most: rows per thread = kNarrowTiles / 2 */>
__global__ __launch_bounds__(256, 4) void k_select_write_narrow(Geom g, int channels, int mode, int relu,
                                                                const int* __restrict__ cand_start,
                                                                const int* __restrict__ tile_start,
                                                                const unsigned* __restrict__ cand_lin,
                                                                const float* __restrict__ resp,
                                                                const ColState* __restrict__ cols,
                                                                unsigned long long* tile_state, Counters* ctr,
                                                                int32_t* __restrict__ out_coords,
                                                                float* __restrict__ out_feats, long long out_capacity,
                                                                long long* __restrict__ nnz_out, long long aux_imm,
                                                                int aux_is_cand, int tps /* tiles per ticket */) {
    constexpr int RPT = kNarrowTiles * kTileRows / 256;  // rows per thread
    __shared__ int s_cnt[RPT * 4];                       // kept rows of each (row group, wave)
    __shared__ int s_ticket;
    __shared__ long long s_base;
    const int n_tiles = (int)ctr->n_tiles;
    const int n_super = (n_tiles + tps - 1) / tps;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const unsigned long long lt_mask = (1ull << lane) - 1ull;
    const bool vec4 = (channels & 3) == 0 && ((size_t)out_feats & 15) == 0;

    for (;;) {
        __syncthreads();  // the previous super-tile's readers of s_ticket / s_base / s_cnt are done
        if (threadIdx.x == 0) s_ticket = (int)take_ticket(ctr, 1u);
        __syncthreads();
        const int st = s_ticket;
        if (st >= n_super) break;
        const bool once = (int)gridDim.x >= n_super;  // one ticket per workgroup covers the layer: do not ask again
        float v[RPT][CMAX];
        bool keep_row[RPT];
        int row_b[RPT], row_first[RPT];
        // row q of the thread: tile st * tps + (q * 256 + threadIdx.x) / 128, local row (.. & 127); the 64
        // rows of a wave always lie in one tile
#pragma unroll
        for (int q = 0; q < RPT; ++q) {
            const int e = q * 256 + threadIdx.x;
            const int tile = st * tps + (e >> 7), r = e & (kTileRows - 1);
            keep_row[q] = false;
            row_b[q] = 0;
            row_first[q] = -1;
            if ((e >> 7) < tps && tile < n_tiles) {  // (uniform in the wave)
                const int b = sample_of_tile(tile_start, g.batch, tile);
                const int first = cand_start[b] + (tile - tile_start[b]) * kTileRows;
                int nrows = cand_start[b + 1] - first;
                if (nrows > kTileRows) nrows = kTileRows;
                const unsigned pos = (unsigned)(tile - tile_start[b]) * kTileRows + (unsigned)r;
                row_b[q] = b;
                if (r < nrows) row_first[q] = first + r;
                const float* seg = resp + (size_t)tile * channels * kTileRows + r;
#pragma unroll
                for (int c = 0; c < CMAX; ++c)
                    if (c < channels) v[q][c] = seg[(size_t)c * kTileRows];
                bool any = false;
#pragma unroll
                for (int c = 0; c < CMAX; ++c) {
                    if (c < channels) {
                        const ColState* cs = cols + (size_t)b * channels + c;
                        const unsigned tau = cs->tau, cut = cs->cut;
                        const float x = v[q][c];
                        const unsigned key = score_key(x, mode);
                        bool keep = key > (pos <= cut ? tau - (tau != 0u ? 1u : 0u) : tau);
                        if (relu) keep = keep && (x > 0.0f);
                        keep = keep && r < nrows;
                        v[q][c] = keep ? x : 0.0f;
                        any |= keep;
                    }
                }
                keep_row[q] = any;
            }
        }
        unsigned long long ball[RPT];
#pragma unroll
        for (int q = 0; q < RPT; ++q) {
            ball[q] = __ballot(keep_row[q]);
            if (lane == 0) s_cnt[q * 4 + wave] = __popcll(ball[q]);
        }
        __syncthreads();
        if (wave == 0) {
            int total = 0;
#pragma unroll
            for (int i = 0; i < RPT * 4; ++i) total += s_cnt[i];
            const long long base = lookback_wave(tile_state, st, total, ctr);
            if (lane == 0) {
                if (st == n_super - 1)
                    __hip_atomic_store(&ctr->n_rows, base + total, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                s_base = base;
            }
        }
        __syncthreads();
        const long long base = s_base;
#pragma unroll
        for (int q = 0; q < RPT; ++q) {
            int before = 0;  // kept rows of the super-tile before this wave's group (groups ascend with q, then wave)
            for (int i = 0; i < q * 4 + wave; ++i) before += s_cnt[i];
            const long long o = base + before + __popcll(ball[q] & lt_mask);
            if (keep_row[q] && o < out_capacity) {
                int c0, c1, c2;
                site_of(g, cand_lin[row_first[q]], c0, c1, c2);
                store_site(g, out_coords + o * (1 + g.ndim), row_b[q], c0, c1, c2);
                float* dst = out_feats + o * channels;
                if (vec4) {
#pragma unroll
                    for (int c = 0; c < CMAX; c += 4)
                        if (c < channels) *(float4*)(dst + c) = make_float4(v[q][c], v[q][c + 1], v[q][c + 2], v[q][c + 3]);
                } else {
#pragma unroll
                    for (int c = 0; c < CMAX; ++c)
                        if (c < channels) dst[c] = v[q][c];
                }
            }
        }
        if (once) break;
    }
    finish_if_last(ctr, nnz_out, aux_imm, aux_is_cand, out_capacity);
}

hipError_t launch_select_write(const Geom& g, int channels, int mode, int relu, const int* cand_start,
                               const int* tile_start, const unsigned* cand_lin, const float* resp,
                               const ColState* cols, unsigned long long* tile_state, long long tiles_cap,
                               Counters* ctr, int32_t* out_coords, float* out_feats, long long out_capacity,
                               long long* nnz_out, long long aux_imm, int aux_is_cand, hipStream_t s) {
    // no more workgroups than can be resident at once (4 per CU by LDS), so that every ticket holder runs; three per
    // CU measured best for the wide kernels (cfg 4: 103 us against 107 with four and 110 with two)
    long long blocks = tiles_cap < 1 ? 1 : (tiles_cap > 256 * 3 ? 256 * 3 : tiles_cap);
    // Narrow layers: a ticket covers 1, 2, 4 .. NT_ tiles, the fewest that leave at most two tickets per CU (a small
    // layer is bound by the tickets, taken one at a time, and every workgroup launched takes at least one; one per
    // CU and four per CU both measured slower on the paper's networks).
#define SCNN_NARROW_CASE(CMAX_, NT_)                                                                              \
    do {                                                                                                          \
        int tps = 1;                                                                                              \
        while (tps < NT_ && tiles_cap > 512ll * tps) tps *= 2;                                                    \
        long long nb = (tiles_cap + tps - 1) / tps;                                                               \
        nb = nb < 1 ? 1 : (nb > 256 * 3 ? 256 * 3 : nb);                                                          \
        hipLaunchKernelGGL((k_select_write_narrow<CMAX_, NT_>), dim3((unsigned)nb), dim3(256), 0, s, g, channels, \
                           mode, relu, cand_start, tile_start, cand_lin, resp, cols, tile_state, ctr, out_coords, \
                           out_feats, out_capacity, nnz_out, aux_imm, aux_is_cand, tps);                          \
    } while (0)
    if (channels <= 4) SCNN_NARROW_CASE(4, 8);
    else if (channels <= 8) SCNN_NARROW_CASE(8, 8);
    else if (channels <= 16) SCNN_NARROW_CASE(16, 8);
    else if (channels <= 32) SCNN_NARROW_CASE(32, 4);
    else if (channels <= 64)
        hipLaunchKernelGGL(k_select_write64, dim3((unsigned)blocks), dim3(256), 0, s, g, channels, mode, relu,
                           cand_start, tile_start, cand_lin, resp, cols, tile_state, ctr, out_coords, out_feats,
                           out_capacity, nnz_out, aux_imm, aux_is_cand);
    else
        hipLaunchKernelGGL(k_select_write, dim3((unsigned)blocks), dim3(256), 0, s, g, channels, mode, relu,
                           cand_start, tile_start, cand_lin, resp, cols, tile_state, ctr, out_coords, out_feats,
                           out_capacity, nnz_out, aux_imm, aux_is_cand);
#undef SCNN_NARROW_CASE
    return hipGetLastError();
}

}  // namespace scnn
