// The attention step (Sec. 3.2; Algorithm 1 steps 13, 15-17): per (sample,
// output channel) keep the k strongest non-zero responses, then compact the
// surviving sites into sorted output rows.
//
// Selection = radix select on an order-preserving 32-bit key of the score, on a
// small part of each column.  A workgroup per column first reads a sample of
// the column (every S-th tile) and brackets the k-th strongest key between two
// of the sample's order statistics.  One pass over the response matrix then
// counts, per column, the entries above the bracket, copies the few percent
// inside it (value and position in the column) to a side buffer, and notes
// which rows hold an entry above the bracket.  A workgroup per column settles
// the rest on the side buffer: the exact k-th largest key tau, the number n_eq
// of entries equal to it and how many of those, q, still fit.  An entry
// survives iff  key > tau, or key == tau and it is among the q equal entries
// of lowest lin; candidate sites are stored in ascending lin, so "lowest lin"
// is "smallest position", and the q-th smallest position among the equal
// entries (a second, ascending radix select on the side buffer) is the cut.
// A bracket that turns out not to hold the k-th entry costs time, never
// exactness: the column is then settled from the response matrix itself.
// The response matrix is read twice in full (the classifying pass, and the
// final mask + compaction + write) and once in a sample of 1/S.  Columns short
// enough for one workgroup's registers are selected in a single launch.
//
// Compaction: where the selection has noted the rows (layers of 33 to 64
// channels), the rows that survive in every tile are known before the last
// pass, a scan gives each tile its first output row, and the write pass
// streams with no ordering between tiles.  Elsewhere tiles are taken in order
// and a tile learns its first output row by looking back at its predecessors.
#include <type_traits>

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
    __shared__ unsigned s_wave[4];
    const int n_tiles = sample_ranges_256(g.batch, cand_start, tile_start, nullptr, s_wave);
    if (threadIdx.x == 0) {
        ctr->n_tiles = n_tiles;
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

// Rank search in a 2048-bin histogram held in LDS.  descending: find the bin holding the kk-th entry counted from
// the top bin; else from the bottom bin.  Returns the bin and the number of entries strictly before it in that
// order.  1 <= kk <= total must hold.  Contains two __syncthreads(); s_res is two shared words that the next call
// must not share (callers alternate between two pairs): the result is read after the last barrier.
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
}

// First launch: a bracket [tau_lo, tau_hi] around the k-th strongest key of every column, from a sample of the
// column.  One workgroup per column reads every S-th tile of it (at most kBracketTiles tiles, whole tiles: 512
// contiguous bytes per channel), keeps the keys in registers and looks up, by two radix digits (22 key bits), the
// sample's keys at the ranks  r -+ delta,  r = k * (sample slots / column slots)  being where the k-th strongest
// entry of the column is expected in the sample (empty slots rank last, as key 0).  delta = 8 standard deviations
// of a uniformly drawn sample's rank plus half a percent of the sample: tiles are pieces of space, not independent
// draws, hence the margin (6 deviations plus a quarter percent missed on three layers of the 128^3 network and on
// the r = 128 layer).  Nothing depends on the bracket being right: the second launch counts what lies above it and
// the third one checks that the k-th entry fell inside, and settles the column from the response matrix itself when
// it did not.
constexpr int kBracketThreads = 1024;
constexpr int kBracketPerThread = 16;
constexpr int kBracketTiles = kBracketThreads * kBracketPerThread / kTileRows;  // 128

__global__ __launch_bounds__(kBracketThreads) void k_bracket(int mode, int channels,
                                                             const int* __restrict__ tile_start,
                                                             const float* __restrict__ resp, long long k,
                                                             ColState* __restrict__ cols) {
    __shared__ unsigned s_h[kHistBins], s_h2[kHistBins];
    __shared__ unsigned s_wave[4];
    __shared__ int s_res[4];
    __shared__ unsigned s_total;
    __shared__ unsigned s_range[2];
    auto clamp_add = [](unsigned a, unsigned c) { return a + c < a ? 0xffffffffu : a + c; };
    const int col = blockIdx.x;
    const int b = col / channels, oc = col - b * channels;
    const int t0 = tile_start[b], t1 = tile_start[b + 1];
    const int T = t1 - t0;
    ColState st;
    st.tau = 0; st.cut = 0xffffffffu; st.n_eq = 0; st.q = 0; st.tau_lo = 1u; st.tau_hi = 0u; st.n_nz = 0; st.n_above = 0;
    st.side_fill = 0; st.done = 0;
    st.side_off = ((unsigned long long)t0 * channels + (unsigned long long)oc * T) * kTileRows;
    if (k <= 0 || T == 0) {
        st.done = 1;
        if (k <= 0) st.tau = 0xffffffffu;  // no key is stronger: nothing survives
        if (threadIdx.x == 0) cols[col] = st;
        return;
    }
    const int S = (T + kBracketTiles - 1) / kBracketTiles;  // every S-th tile
    const int ns_tiles = (T + S - 1) / S;
    const unsigned m_s = (unsigned)ns_tiles * kTileRows;
    if (threadIdx.x == 0) {
        s_total = 0;
        s_range[0] = 0xffffffffu;
        s_range[1] = 0u;
    }
    unsigned key[kBracketPerThread];
    unsigned mine = 0;
#pragma unroll
    for (int u = 0; u < kBracketPerThread; ++u) {
        const unsigned i = (unsigned)u * kBracketThreads + threadIdx.x;
        key[u] = 0u;
        if (i < m_s)
            key[u] = score_key(resp[((size_t)(t0 + (int)(i >> 7) * S) * channels + oc) * kTileRows + (i & 127u)], mode);
        mine += key[u] != 0u ? 1u : 0u;
    }
    // the sample's entries, and the range of their keys
    unsigned kmin = 0xffffffffu, kmax = 0u;
#pragma unroll
    for (int u = 0; u < kBracketPerThread; ++u) {
        if (key[u] != 0u) {
            kmin = key[u] < kmin ? key[u] : kmin;
            kmax = key[u] > kmax ? key[u] : kmax;
        }
    }
    __syncthreads();  // (s_total and the range words are set up)
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        mine += __shfl_xor(mine, d, 64);
        const unsigned a = __shfl_xor(kmin, d, 64), c = __shfl_xor(kmax, d, 64);
        kmin = a < kmin ? a : kmin;
        kmax = c > kmax ? c : kmax;
    }
    if ((threadIdx.x & 63) == 0 && mine) {
        atomicAdd(&s_total, mine);
        atomicMin(&s_range[0], kmin);
        atomicMax(&s_range[1], kmax);
    }
    __syncthreads();
    const long long nz = (long long)s_total;
    kmin = s_range[0];
    kmax = s_range[1];
    const double r = (double)k * (double)m_s / ((double)T * kTileRows);
    const double frac = r / (double)m_s;
    double delta = 0.0;  // (a sample of every tile is the column: the ranks are exact)
    if (S > 1) delta = 8.0 * sqrt(r * (frac < 1.0 ? 1.0 - frac : 0.0)) + 0.005 * (double)m_s + 16.0;
    const double r_up = floor(r - delta), r_dn = ceil(r + delta);
    // The sample's keys at ranks r_up and r_dn (1 = strongest), cut down to two digits of 11 bits.  The digits are
    // taken from key - kmin: the leading bits of the keys themselves are the same for most of a column (sign, high
    // exponent bits), and a histogram whose entries fall into a dozen bins is a queue at those LDS words.  Past the
    // sample's entries on the strong side nothing is above the bracket; past them on the weak side every entry is in
    // it or above it.
    const bool want_up = r_up >= 1.0 && (long long)r_up <= nz, want_dn = r_dn >= 1.0 && r_dn <= (double)nz;  // (uniform)
    long long rank_up = want_up ? (long long)r_up : 1, rank_dn = want_dn ? (long long)r_dn : 1;
    const unsigned span = nz > 0 ? kmax - kmin : 0u;
    const int nb = span ? 32 - __clz(span) : 1;  // bits of key - kmin
    const int sh1 = nb > 11 ? nb - 11 : 0;       // first digit: bits [sh1, nb)
    const int sh2 = sh1 > 11 ? sh1 - 11 : 0;     // second digit: bits [sh2, sh1)
    const unsigned mask2 = (1u << (sh1 - sh2)) - 1u;
    for (int i = threadIdx.x; i < kHistBins; i += kBracketThreads) s_h[i] = 0;
    __syncthreads();
#pragma unroll
    for (int u = 0; u < kBracketPerThread; ++u)
        if (key[u] != 0u) atomicAdd(&s_h[(key[u] - kmin) >> sh1], 1u);
    __syncthreads();
    int bin_up = 0, bin_dn = 0;
    unsigned before = 0;
    if (nz > 0) {
        block_pick(s_h, rank_up, true, s_wave, s_res, bin_up, before);
        rank_up -= (long long)before;
        block_pick(s_h, rank_dn, true, s_wave, s_res + 2, bin_dn, before);
        rank_dn -= (long long)before;
    }
    int sub_up = 0, sub_dn = 0;
    if (sh1 > 0) {  // (uniform)
        for (int i = threadIdx.x; i < kHistBins; i += kBracketThreads) {
            s_h[i] = 0;
            s_h2[i] = 0;
        }
        __syncthreads();
#pragma unroll
        for (int u = 0; u < kBracketPerThread; ++u) {
            if (key[u] == 0u) continue;
            const unsigned d = key[u] - kmin;
            if ((int)(d >> sh1) == bin_up) atomicAdd(&s_h[(d >> sh2) & mask2], 1u);
            if ((int)(d >> sh1) == bin_dn) atomicAdd(&s_h2[(d >> sh2) & mask2], 1u);
        }
        __syncthreads();
        if (nz > 0) {
            block_pick(s_h, rank_up, true, s_wave, s_res, sub_up, before);
            block_pick(s_h2, rank_dn, true, s_wave, s_res + 2, sub_dn, before);
        }
    }
    st.tau_hi = 0xffffffffu;  // rank < 1: nothing is above
    if (r_up >= 1.0)  // (the upper end of the two-digit bin)
        st.tau_hi =
            want_up ? clamp_add(kmin, ((unsigned)bin_up << sh1) | ((unsigned)sub_up << sh2) | ((1u << sh2) - 1u)) : 0u;
    if (want_dn) {
        const unsigned lo = kmin + (((unsigned)bin_dn << sh1) | ((unsigned)sub_dn << sh2));
        st.tau_lo = lo ? lo : 1u;
    }
    if (threadIdx.x == 0) cols[col] = st;
}

// Second launch, grid = (sample x group of kClassifyWaves channels, slices); a wave per channel, the waves of a
// workgroup on the same tiles (adjacent channels of a tile are adjacent in memory).  Counts the column's entries and
// those above the bracket, copies the entries inside it (value and position in the column) to the side buffer, and,
// when row_plane is given, records which rows hold an entry above the bracket -- those survive whatever the exact
// threshold turns out to be -- in the channel's own plane of row marks, two 64-bit words per tile, which
// k_combine_marks merges.  Waves share nothing but the cursor of their column's side-buffer entries and never wait
// for one another.  (Marks kept in one shared plane cost 40 us of device-scope atomics on the r = 128 layer, whose
// every tile half would be updated by every channel.)  The loop is bound by
// instruction issue, hence the float compares on ballots, the counts in scalar registers and the marks gathered
// with v_writelane.
// With the score s(x) = |x| or x: the value t such that, for an entry x (non-zero, not a NaN),
// score_key(x) > key  <=>  s(x) > t  and  score_key(x) >= key  <=>  s(x) >= t:  the float whose key `key` is, or, for the
// keys below every float's (signed order: 0 .. 0x007fffff), minus infinity.  Key 0xffffffff gives a NaN: no score
// compares above it.
__device__ inline float score_bound(unsigned key, int mode) {
    if (mode == SCNN_TOPK_ABS) return __uint_as_float(key);  // (keys are the bit patterns of |x|; key 0 is 0.0)
    if (key >= 0x80000000u) return __uint_as_float(key & 0x7fffffffu);
    return key <= 0x007fffffu ? -INFINITY : __uint_as_float(~key);
}

// lo and hi with lane `lane` (a constant once the loops are unrolled) replaced by the halves of the lane mask m.  The
// mask is copied by scalar moves first: it may come straight from a vector compare, and a lane write that reads a
// scalar register too soon after a vector instruction wrote it gets the old contents; the compiler, which keeps
// that distance for its own instructions, does not look inside an asm statement (and has no builtin for the lane
// write here).  A scalar move waits for the vector instruction by itself.
__device__ inline void write_lanes(unsigned& lo, unsigned& hi, unsigned long long m, int lane) {
    unsigned t0, t1;
    asm("s_mov_b32 %2, %4\n\ts_mov_b32 %3, %5\n\tv_writelane_b32 %0, %2, %6\n\tv_writelane_b32 %1, %3, %6"
        : "+v"(lo), "+v"(hi), "=&s"(t0), "=&s"(t1)
        : "s"((unsigned)m), "s"((unsigned)(m >> 32)), "i"(lane));
}

constexpr int kClassifyWaves = 8;
constexpr int kClassifyTiles = 4;
constexpr int kClassifyStage = 768;  // entries staged per wave (640, four workgroups per CU, measured the same)
constexpr int kClassifySlicesMax = 256;  // (the third launch scans a column's slices with its first 256 threads)

// Tiles per slice when a column of T tiles is cut into `slices` runs of whole iterations.
__host__ __device__ inline int classify_slice_tiles(int T, int slices) {
    const int per = (T + slices - 1) / slices;
    return (per + kClassifyTiles - 1) / kClassifyTiles * kClassifyTiles;
}

template <int MODE, bool MARKS /* row_plane given: the rows of sure survivors are recorded */>
__global__ __launch_bounds__(kClassifyWaves * 64) void k_classify(int relu, int channels,
                                                                  const int* __restrict__ tile_start,
                                                                  const float* __restrict__ resp,
                                                                  ColState* __restrict__ cols,
                                                                  uint2* __restrict__ side, uint2* __restrict__ part,
                                                                  unsigned long long* __restrict__ row_plane,
                                                                  long long plane_words) {
    constexpr int U = kClassifyTiles;  // tiles per iteration
    constexpr int WCAP = kClassifyStage;  // staged entries per wave (a flush leaves room for an iteration's worth)
    __shared__ uint2 s_buf[kClassifyWaves * WCAP];
    const int groups = (channels + kClassifyWaves - 1) / kClassifyWaves;
    const int b = blockIdx.x / groups;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // (uniform, and known to be)
    const int oc = (blockIdx.x - b * groups) * kClassifyWaves + wave;
    if (oc >= channels) return;  // (the last group may be short)
    const int col = b * channels + oc;
    const ColState st = cols[col];
    if (st.done) return;
    const int t0 = tile_start[b], t1 = tile_start[b + 1];
    const float s_lo = score_bound(st.tau_lo, MODE), s_hi = score_bound(st.tau_hi, MODE);
    const unsigned long long relu_off = relu ? 0ull : ~0ull;
    // |x| as the score: a row survives for sure when y > sure_hi, y = x under ReLU (a negative value is dropped
    // later), |x| without; sure_hi = the bracket's upper end where that is a number not below zero (an entry above it
    // is then non-zero, and positive under ReLU), 0 where it is negative (every entry is above it), infinity where it
    // is no number (no entry compares above it)
    const unsigned sure_sign = relu ? 0xffffffffu : 0x7fffffffu;
    const float sure_hi = s_hi >= 0.0f ? s_hi : (s_hi < 0.0f ? 0.0f : INFINITY);
    uint2* wbuf = s_buf + wave * WCAP;
    int fill = 0;                    // wave-uniform
    unsigned n_nz = 0, n_above = 0;  // per lane
    // slice y of the column: tiles [first, last)
    const int L = classify_slice_tiles(t1 - t0, (int)gridDim.y);
    const int first = t0 + (int)blockIdx.y * L;
    const int last = first + L < t1 ? first + L : t1;
    // a flush reserves its piece of the column's side-buffer entries from the column's cursor: one returning atomic
    // per wave and flush, a few thousand a layer, which is what keeps the column's entries in one run
    uint2* run = side + st.side_off;
    auto flush = [&]() {
        unsigned base = 0;
        if (lane == 0) base = atomicAdd(&cols[col].side_fill, (unsigned)fill);
        base = __builtin_amdgcn_readfirstlane(base);
        for (int i = lane; i < fill; i += 64) run[base + i] = wbuf[i];
        fill = 0;
    };
    unsigned long long* plane = MARKS ? row_plane + (size_t)oc * plane_words : nullptr;
    // the values of tiles tile0 .. tile0 + U - 1 at rows lane and lane + 64 (a tile past the slice: the slice's first)
    auto load = [&](int tile0, float (&v)[U][2]) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int tile = tile0 + u;
            const float* seg = resp + ((size_t)(tile < last ? tile : first) * channels + oc) * kTileRows;
            v[u][0] = seg[lane];
            v[u][1] = seg[64 + lane];
        }
    };
    // one iteration: the tiles tile0 .. tile0 + U - 1, whose values are in v; FULL: all of them are in the slice.
    // The loop is bound by scalar instructions (lane masks are combined, counted and turned into branch conditions
    // there), so whatever can be decided per lane is: the two counts are kept per lane and added up at the end,
    // the bracket test is one condition whose mask is also the staging order, and with |x| as the score the rows
    // that survive for sure are one compare (x, or |x| without ReLU, against the bracket's upper end).
    auto process = [&](int tile0, const float (&v)[U][2], auto full) {
        constexpr bool FULL = decltype(full)::value;
        unsigned mark_lo = 0, mark_hi = 0;  // lane j: the marks of tile j / 2, rows (j & 1) * 64 ..
        const unsigned pos0 = (unsigned)(tile0 - t0) * kTileRows + (unsigned)lane;
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const float x = (FULL || tile0 + u < last) ? v[u][h] : 0.0f;
                const float sc = MODE == SCNN_TOPK_ABS ? fabsf(x) : x;
                const bool nz = x != 0.0f, above = nz && sc > s_hi;
                const bool hit = nz && sc >= s_lo && !(sc > s_hi);  // inside the bracket
                const unsigned long long m = __ballot(hit);
                n_nz += nz ? 1u : 0u;
                n_above += above ? 1u : 0u;
                if constexpr (MARKS) {
                    unsigned long long sure;
                    if constexpr (MODE == SCNN_TOPK_ABS)
                        sure = __ballot(__uint_as_float(__float_as_uint(x) & sure_sign) > sure_hi);
                    else
                        sure = __ballot(above) & (__ballot(x > 0.0f) | relu_off);
                    write_lanes(mark_lo, mark_hi, sure, u * 2 + h);
                }
                if (hit) {  // the value itself is staged; its key is taken when the entry is read
                    const unsigned rank =
                        __builtin_amdgcn_mbcnt_hi((unsigned)(m >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)m, 0u));
                    wbuf[fill + (int)rank] = make_uint2(__float_as_uint(x), pos0 + (unsigned)(u * kTileRows + h * 64));
                }
                fill += __popcll(m);
            }
        }
        if (MARKS && lane < 2 * U && (FULL || tile0 + (lane >> 1) < last))
            plane[2 * (size_t)tile0 + lane] = ((unsigned long long)mark_hi << 32) | mark_lo;
    };
    auto process_any = [&](int tile0, const float (&v)[U][2]) {
        if (tile0 + U <= last) process(tile0, v, std::true_type{});
        else process(tile0, v, std::false_type{});
    };
    // Two register sets in turn, so that an iteration's loads are in flight during the whole of the one before it.
    // The staging buffer is emptied, when an iteration could overfill it, before the next loads are issued, never
    // between an iteration's loads and their use, and the next loads are issued whether or not there is a next
    // iteration: the compiler counts outstanding loads along every path, and behind a loop of stores, or a branch
    // that may have skipped the loads, it waits for all of them.
    auto make_room = [&]() {
        if (fill > WCAP - U * kTileRows) flush();
    };
    float va[U][2], vb[U][2];
    if (first < last) load(first, va);
    for (int tile0 = first; tile0 < last; tile0 += 2 * U) {
        make_room();
        load(tile0 + U, vb);  // (always: past the slice it reads the slice's first tile again, and nobody looks)
        process_any(tile0, va);
        if (tile0 + U >= last) break;
        make_room();
        load(tile0 + 2 * U, va);
        process_any(tile0 + U, vb);
    }
    if (fill > 0) flush();
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        n_nz += __shfl_xor(n_nz, d, 64);
        n_above += __shfl_xor(n_above, d, 64);
    }
    if (lane == 0) part[(size_t)col * gridDim.y + blockIdx.y] = make_uint2(n_nz, n_above);
}

// Third launch, one workgroup per column: the exact k-th strongest key tau, the number of entries equal to it and,
// if those do not all fit, the position up to which they do -- by radix select over the column's side-buffer
// entries when the bracket held the k-th entry (the rule), over the column itself when it did not.
constexpr int kSideThreads = 1024;

struct SideEntries {  // entry i of a column's side-buffer entries: {key, position}; the buffer holds the value's bits
    const uint2* e;
    int mode;
    __device__ uint2 operator()(unsigned i) const {
        const uint2 x = e[i];
        return make_uint2(score_key(__uint_as_float(x.x), mode), x.y);
    }
};
struct ColumnEntries {  // slot i of a column of the response matrix (key 0: not an entry)
    const float* col;   // the column's values in its first tile
    size_t tile_pitch;  // floats from one tile to the next
    int mode;
    __device__ uint2 operator()(unsigned i) const {
        return make_uint2(score_key(col[(size_t)(i >> 7) * tile_pitch + (i & 127u)], mode), i);
    }
};

// tau = the kk-th strongest key among m entries {key, position} whose keys lie in [key_lo, key_hi] (key 0: not an
// entry); n_eq entries equal it, the q of lowest position survive: those at positions <= cut.  1 <= kk <= number of
// entries.  The digits of the radix select, 11 bits at most, are taken from key - key_lo, most significant first, so
// that a narrow bracket is settled in two passes.  Between the passes up to kSettleCached entries per thread are held
// in registers and kSettleLds more per workgroup in LDS (brackets that hold long runs of equal scores run to 30 000
// entries on the paper's first layers).  (whole workgroup)
// Two sizes: 20 per thread + 12288 (one workgroup per compute unit: its registers and LDS), the rule; 4 per thread +
// 2048 for layers of many columns, whose brackets are short and whose workgroups then fit two to a compute unit.
template <int kSettleCached> constexpr unsigned kSettleRegsOf = (unsigned)kSettleCached * 1024u;

// held: the entries threadIdx.x + 1024 * u of the column, more: the entries from kSettleRegs on, if cached
// (m <= kSettleRegs + kSettleLds); both loaded by the caller.
template <int kSettleCached, class Entries>
__device__ inline void settle_column(const Entries& entry, unsigned m, const uint2 (&held)[kSettleCached],
                                     const uint2* more, bool cached, unsigned key_lo, unsigned key_hi, long long kk,
                                     unsigned* s_h, unsigned* s_wave, int* s_res, unsigned& tau, unsigned& n_eq,
                                     unsigned& q, unsigned& cut) {
    constexpr unsigned kSettleRegs = kSettleRegsOf<kSettleCached>;
    auto clear = [&]() {
        for (int i = threadIdx.x; i < kHistBins; i += kSideThreads) s_h[i] = 0;
        __syncthreads();
    };
    // Data with long runs of equal scores (unit input values) sends most lanes of a wave to one bin, and LDS serves
    // the atomics of a wave on one word one after the other: the lanes that share the first active lane's bin add
    // once, through that lane; the others add on their own.
    auto add = [&](bool valid, unsigned bin) {
        const unsigned long long act = __ballot(valid);
        if (act == 0ull) return;  // (uniform)
        const int first = __ffsll((long long)act) - 1;
        const unsigned b0 = __shfl(valid ? bin : 0u, first, 64);
        const unsigned long long same = __ballot(valid && bin == b0);
        if ((int)(threadIdx.x & 63) == first) atomicAdd(&s_h[b0], (unsigned)__popcll(same));
        else if (valid && bin != b0) atomicAdd(&s_h[bin], 1u);
    };
    // histogram of digit(entry) over the entries that pass(entry)
    auto histogram = [&](auto pass, auto digit) {
        clear();
        if (cached) {
#pragma unroll
            for (int u = 0; u < kSettleCached; ++u) {
                const bool valid = held[u].x != 0u && pass(held[u]);
                add(valid, valid ? digit(held[u]) : 0u);
            }
            if (m > kSettleRegs) {  // (uniform; whole waves take part in every round: add() uses ballots)
                const unsigned n_more = m - kSettleRegs;
                for (unsigned j0 = 0; j0 < n_more; j0 += kSideThreads) {
                    const unsigned j = j0 + threadIdx.x;
                    const uint2 x = j < n_more ? more[j] : make_uint2(0u, 0u);
                    const bool valid = x.x != 0u && pass(x);
                    add(valid, valid ? digit(x) : 0u);
                }
            }
        } else {
            for (unsigned i0 = threadIdx.x; i0 < m; i0 += kSideThreads * 8) {  // loads issued eight at a time
                uint2 x[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const unsigned i = i0 + (unsigned)kSideThreads * u;
                    x[u] = i < m ? entry(i) : make_uint2(0u, 0u);
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const bool valid = x[u].x != 0u && pass(x[u]);
                    add(valid, valid ? digit(x[u]) : 0u);
                }
            }
        }
        __syncthreads();
    };
    int bin = 0, picks = 0;
    unsigned before = 0;
    const unsigned span = key_hi - key_lo;
    int nb = span ? 32 - __clz(span) : 1;  // bits of key - key_lo still open
    unsigned prefix = 0;                   // the bits above them
    while (nb > 0) {
        const int w = nb < 11 ? nb : 11, shift = nb - w;
        const int above = nb;  // (captured by value)
        histogram([=](uint2 x) { return (unsigned)((unsigned long long)(x.x - key_lo) >> above) == prefix; },
                  [=](uint2 x) { return ((x.x - key_lo) >> shift) & ((1u << w) - 1u); });
        block_pick(s_h, kk, true, s_wave, s_res + 2 * (picks++ & 1), bin, before);
        kk -= (long long)before;
        prefix = (prefix << w) | (unsigned)bin;
        nb = shift;
    }
    tau = key_lo + prefix;
    n_eq = s_h[bin];
    q = (unsigned)kk;  // 1 <= q <= n_eq
    __syncthreads();
    cut = 0xffffffffu;
    if (q < n_eq) {
        // q-th smallest position among the entries equal to tau: ascending radix select on the position
        const unsigned t = tau;
        unsigned pprefix = 0;
        long long rank = q;
        for (int pass = 0; pass < 3; ++pass) {
            const int shift = pass == 0 ? 21 : (pass == 1 ? 10 : 0), bits = pass == 2 ? 10 : 11;
            histogram([=](uint2 x) { return x.x == t && (pass == 0 || (x.y >> (shift + bits)) == pprefix); },
                      [=](uint2 x) { return (x.y >> shift) & ((1u << bits) - 1u); });
            block_pick(s_h, rank, false, s_wave, s_res + 2 * (picks++ & 1), bin, before);
            pprefix = (pprefix << bits) | (unsigned)bin;
            rank -= (long long)before;
        }
        cut = pprefix;
    }
}

template <int kSettleCached, unsigned kSettleLds>
__global__ __launch_bounds__(kSideThreads) __attribute__((amdgpu_waves_per_eu(kSettleCached > 8 ? 4 : 8)))
void k_settle(int mode, int relu, int channels, long long k,
                                                         const int* __restrict__ tile_start,
                                                         const float* __restrict__ resp, ColState* __restrict__ cols,
                                                         const uint2* __restrict__ side,
                                                         const uint2* __restrict__ part, int slices,
                                                         unsigned long long* row_keep,
                                                         long long* __restrict__ tile_base, Counters* ctr) {
    __shared__ unsigned s_h[kHistBins];
    __shared__ unsigned s_wave[4];
    __shared__ int s_res[4];
    __shared__ uint2 s_part[4];
    constexpr unsigned kSettleRegs = kSettleRegsOf<kSettleCached>;
    __shared__ uint2 s_more[kSettleLds];
    __shared__ unsigned s_cnt;
    const int col = blockIdx.x;
    const int b = col / channels, oc = col - b * channels;
    const int t0 = tile_start[b], t1 = tile_start[b + 1];
    ColState st = cols[col];
    // the slices' counts of entries and of entries above the bracket (read along with the column's state; unused, and
    // possibly stale, where the column is settled already)
    uint2 my_part = make_uint2(0u, 0u);
    if ((int)threadIdx.x < slices) my_part = part[(size_t)col * slices + threadIdx.x];
    if (!st.done) {
        unsigned sum_nz = my_part.x, sum_above = my_part.y;
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) {
            sum_nz += __shfl_xor(sum_nz, d, 64);
            sum_above += __shfl_xor(sum_above, d, 64);
        }
        if (threadIdx.x < 256 && (threadIdx.x & 63) == 0) s_part[threadIdx.x >> 6] = make_uint2(sum_nz, sum_above);
        __syncthreads();
        st.n_nz = s_part[0].x + s_part[1].x + s_part[2].x + s_part[3].x;
        st.n_above = s_part[0].y + s_part[1].y + s_part[2].y + s_part[3].y;
        const unsigned m = st.side_fill;
        const float* col0 = resp + ((size_t)t0 * channels + oc) * kTileRows;
        const size_t pitch = (size_t)channels * kTileRows;
        const SideEntries e{side + st.side_off, mode};
        // the side buffer's entries of the column, in registers if they are few enough (the rule)
        const bool cached = m <= kSettleRegs + kSettleLds;  // (uniform)
        uint2 kept[kSettleCached];
        if (cached) {
#pragma unroll
            for (int u = 0; u < kSettleCached; ++u) {
                const unsigned i = threadIdx.x + (unsigned)kSideThreads * u;
                kept[u] = i < m ? e(i) : make_uint2(0u, 0u);
            }
            for (unsigned i = kSettleRegs + threadIdx.x; i < m; i += kSideThreads) s_more[i - kSettleRegs] = e(i);
            __syncthreads();
        }
        // the row of a surviving entry of the bracket is marked unless some channel has marked it already
        auto word_of = [&](uint2 x) { return row_keep + 2 * (size_t)(t0 + (int)(x.y >> 7)) + ((x.y >> 6) & 1u); };
        auto mark = [&](uint2 x, unsigned long long have) {
            const unsigned long long bit = 1ull << (x.y & 63u);
            if (have & bit) return;
            if (relu && !(col0[(size_t)(x.y >> 7) * pitch + (x.y & 127u)] > 0.0f)) return;
            atomicOr(word_of(x), bit);
        };
        unsigned m_eff = m;        // the entries the marking below runs over, and whether they are the cached ones
        bool cached_eff = cached;
        bool held;  // the side buffer decides the column
        if ((long long)st.n_nz <= k) {
            // fewer entries than k: all survive (tau = 0, every non-zero key is above it); the rows are all marked if
            // no entry lay below the bracket
            st.tau = 0;
            held = st.n_above + m == st.n_nz;
        } else {
            const long long k_rem = k - (long long)st.n_above;
            held = k_rem >= 1 && k_rem <= (long long)m;
            bool settled = false;
            if (held && !cached) {
                // A bracket too long to cache (few, very long columns): read it twice instead of once per digit.
                // First the histogram of the leading digit; then, with the k-th key's bin known, the entries of that
                // bin go to LDS and the entries above it, which survive whatever the rest of the key, mark their
                // rows; the remaining digits and the tie cut are settled on the cached bin.
                const unsigned span = st.tau_hi - st.tau_lo;
                const int nb = span ? 32 - __clz(span) : 1;
                const int w = nb < 11 ? nb : 11, shift = nb - w;
                const unsigned lo = st.tau_lo;
                auto digit = [=](uint2 x) { return ((x.x - lo) >> shift) & ((1u << w) - 1u); };
                for (int i = threadIdx.x; i < kHistBins; i += kSideThreads) s_h[i] = 0;
                if (threadIdx.x == 0) s_cnt = 0;
                __syncthreads();
                for (unsigned i0 = threadIdx.x; i0 < m; i0 += kSideThreads * 8) {  // eight entries in flight per thread
                    uint2 x[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const unsigned i = i0 + (unsigned)kSideThreads * u;
                        x[u] = i < m ? e(i) : make_uint2(0u, 0u);
                    }
#pragma unroll
                    for (int u = 0; u < 8; ++u)
                        if (x[u].x != 0u) atomicAdd(&s_h[digit(x[u])], 1u);
                }
                __syncthreads();
                int bin;
                unsigned before;
                block_pick(s_h, k_rem, true, s_wave, s_res + 2, bin, before);
                const unsigned in_bin = s_h[bin];
                __syncthreads();  // (every thread has read the count before the histogram is cleared again)
                if (in_bin <= kSettleLds) {  // (uniform)
                    for (unsigned i0 = threadIdx.x; i0 < m; i0 += kSideThreads * 8) {
                        uint2 x[8];
                        unsigned long long have[8];
#pragma unroll
                        for (int u = 0; u < 8; ++u) {
                            const unsigned i = i0 + (unsigned)kSideThreads * u;
                            x[u] = i < m ? e(i) : make_uint2(0u, 0u);
                        }
#pragma unroll
                        for (int u = 0; u < 8; ++u) {
                            have[u] = ~0ull;
                            if (row_keep && x[u].x != 0u && (int)digit(x[u]) > bin)
                                have[u] = __hip_atomic_load(word_of(x[u]), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        }
#pragma unroll
                        for (int u = 0; u < 8; ++u) {
                            if (x[u].x == 0u) continue;
                            const int d = (int)digit(x[u]);
                            if (d == bin) s_more[atomicAdd(&s_cnt, 1u)] = x[u];
                            else if (row_keep && d > bin) mark(x[u], have[u]);
                        }
                    }
#pragma unroll
                    for (int u = 0; u < kSettleCached; ++u) kept[u] = make_uint2(0u, 0u);
                    __syncthreads();
                    const unsigned long long lo2 = (unsigned long long)lo + ((unsigned long long)(unsigned)bin << shift);
                    unsigned long long hi2 = lo2 + ((1ull << shift) - 1ull);
                    if (hi2 > st.tau_hi) hi2 = st.tau_hi;
                    m_eff = kSettleRegs + in_bin;  // (the first kSettleRegs entries are the empty registers)
                    cached_eff = true;
                    settle_column<kSettleCached>(e, m_eff, kept, s_more, true, (unsigned)lo2, (unsigned)hi2, k_rem - (long long)before, s_h,
                                  s_wave, s_res, st.tau, st.n_eq, st.q, st.cut);
                    settled = true;
                }
            }
            if (settled) {
            } else if (held)
                settle_column<kSettleCached>(e, m, kept, s_more, cached, st.tau_lo, st.tau_hi, k_rem, s_h, s_wave, s_res, st.tau, st.n_eq,
                              st.q, st.cut);
            else
                settle_column<kSettleCached>(ColumnEntries{col0, pitch, mode}, (unsigned)(t1 - t0) * kTileRows, kept, s_more, false, 0u,
                              0xffffffffu, k, s_h, s_wave, s_res, st.tau, st.n_eq, st.q, st.cut);
        }
        if (threadIdx.x == 0) {
            st.done = 1;
            cols[col] = st;
            if (!held) atomicOr(&ctr->bracket_failed, 1u);  // the rows marked so far cannot be relied on
        }
        if (row_keep && held) {
            // the bracket's entries that survive keep their rows too
            auto survives = [&](uint2 x) { return x.x > st.tau || (x.x == st.tau && x.x != 0u && x.y <= st.cut); };
            if (cached_eff) {
#pragma unroll
                for (int u0 = 0; u0 < kSettleCached; u0 += 8) {  // eight words in flight per thread
                    unsigned long long have[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        have[u] = ~0ull;
                        if (u0 + u < kSettleCached && survives(kept[u0 + u]))
                            have[u] = __hip_atomic_load(word_of(kept[u0 + u]), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
#pragma unroll
                    for (int u = 0; u < 8; ++u)
                        if (u0 + u < kSettleCached) mark(kept[u0 + u], have[u]);
                }
                for (unsigned i = kSettleRegs + threadIdx.x; i < m_eff; i += kSideThreads) {
                    const uint2 x = s_more[i - kSettleRegs];
                    if (survives(x)) mark(x, __hip_atomic_load(word_of(x), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
                }
            } else {
                for (unsigned i0 = threadIdx.x; i0 < m_eff; i0 += kSideThreads * 8) {  // eight entries in flight per thread
                    uint2 x[8];
                    unsigned long long have[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const unsigned i = i0 + (unsigned)kSideThreads * u;
                        x[u] = i < m_eff ? e(i) : make_uint2(0u, 0u);
                    }
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        have[u] = ~0ull;
                        if (survives(x[u]))
                            have[u] = __hip_atomic_load(word_of(x[u]), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
#pragma unroll
                    for (int u = 0; u < 8; ++u) mark(x[u], have[u]);
                }
            }
        }
    }
    if (!tile_base) return;
    // The workgroup that ends last turns the marked rows into the output row at which every tile starts.  The marks
    // are only ever touched by device-scope atomics, which are performed at the point of coherence; the barrier waits
    // for this workgroup's to be acknowledged, so no cache write-back (a fence, tens of microseconds here) is needed
    // before the count.
    __syncthreads();
    if (threadIdx.x == 0) s_res[0] = (atomicAdd(&ctr->cols_done, 1u) == gridDim.x - 1) ? 1 : 0;
    __syncthreads();
    if (!s_res[0]) return;
    if (__hip_atomic_load(&ctr->bracket_failed, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) return;
    const int n_tiles = (int)ctr->n_tiles;
    const int per = (n_tiles + kSideThreads - 1) / kSideThreads;  // consecutive tiles per thread
    const int first = threadIdx.x * per;
    auto rows_of = [&](int t) -> unsigned {
        return (unsigned)(__popcll(__hip_atomic_load(&row_keep[2 * (size_t)t], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) +
                          __popcll(__hip_atomic_load(&row_keep[2 * (size_t)t + 1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)));
    };
    constexpr int kKept = 8;  // counts held in registers between the two sweeps
    unsigned cnt[kKept];
    unsigned local = 0;
#pragma unroll
    for (int j = 0; j < kKept; ++j) {
        const int t = first + j;
        cnt[j] = (j < per && t < n_tiles) ? rows_of(t) : 0u;
        local += cnt[j];
    }
    for (int t = first + kKept; t < first + per && t < n_tiles; ++t) local += rows_of(t);
    // exclusive scan over the 1024 threads (64-bit sums through s_h)
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    unsigned long long inc = local;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const unsigned long long t = __shfl_up(inc, d, 64);
        if (lane >= d) inc += t;
    }
    unsigned long long* s_tot = (unsigned long long*)s_h;
    __syncthreads();
    if (lane == 63) s_tot[wave] = inc;
    __syncthreads();
    unsigned long long base = 0, total = 0;
    for (int w = 0; w < kSideThreads / 64; ++w) {
        const unsigned long long x = s_tot[w];
        if (w < wave) base += x;
        total += x;
    }
    long long run = (long long)(base + inc - local);
#pragma unroll
    for (int j = 0; j < kKept; ++j) {
        const int t = first + j;
        if (j < per && t < n_tiles) tile_base[t] = run;
        run += cnt[j];
    }
    for (int t = first + kKept; t < first + per && t < n_tiles; ++t) {
        tile_base[t] = run;
        run += rows_of(t);
    }
    if (threadIdx.x == 0) ctr->n_rows = (long long)total;
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
    __shared__ int s_res[4];
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
    st.tau = 0; st.cut = 0xffffffffu; st.n_eq = 0; st.q = 0; st.tau_lo = 0; st.tau_hi = 0; st.n_nz = s_total;
    st.n_above = 0; st.side_fill = 0; st.done = 1; st.side_off = 0;
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
    block_pick(s_h, k_rem, true, s_wave, s_res + 2, bin, before);  // key bits [20:10]
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
        block_pick(s_h, (long long)q, false, s_wave, s_res + 2, bin, before);
        const unsigned phi = (unsigned)bin;
        const long long rank = (long long)q - (long long)before;
        histogram([tau, phi](unsigned x, unsigned i) { return x == tau && (i >> 4) == phi; },
                  [](unsigned, unsigned i) { return i & 15u; });
        block_pick(s_h, rank, false, s_wave, s_res, bin, before);
        cut = (phi << 4) | (unsigned)bin;
    }
    if (threadIdx.x == 0) {
        st.tau = tau;
        st.n_eq = n_eq;
        st.q = q;
        st.cut = cut;
        cols[col] = st;
    }
}

// The same for columns of at most 1024 positions (eight tiles: 2-D grids up to 32 x 32, 3-D up to 10^3), one WAVE
// per column and no shared memory: batches of thousands of such samples (a batch of small images) have thousands
// of columns, and a workgroup of 1024 threads with five passes over a 2048-bin histogram costs each of them about
// 10 us.  The k-th strongest key is found bit by bit, from the top: with the bits above already fixed, the keys
// that have the next bit set are counted (a ballot per register); the tie cut is the position of the q-th equal key
// in position order.  kTinyPerLane = 64 takes columns of up to 4096 positions (16^3 grids).  Both forms are used
// when there are a thousand columns or more; with few columns a workgroup per column is as fast or a little faster
// (the 32 dependent bit steps of a wave against five histogram passes of a workgroup).
constexpr long long kTinyColumn = 64 * 16;   // positions of a column at most, 16 keys per lane
constexpr long long kTinyColumn64 = 64 * 64;  // ... 64 keys per lane
constexpr int kTinyManyColumns = 1024;

template <int kTinyPerLane>
__global__ __launch_bounds__(256) void k_select_tiny(int mode, int channels, int ncols,
                                                     const int* __restrict__ tile_start,
                                                     const float* __restrict__ resp, long long k,
                                                     ColState* __restrict__ cols) {
    const int lane = threadIdx.x & 63;
    const int col = (int)blockIdx.x * 4 + (int)(threadIdx.x >> 6);
    if (col >= ncols) return;  // (whole waves)
    const int b = col / channels, oc = col - b * channels;
    const int t0 = tile_start[b], t1 = tile_start[b + 1];
    const unsigned n = (unsigned)(t1 - t0) * kTileRows;  // positions of the column (<= 64 kTinyPerLane, see the launcher)
    // key u of the lane sits at position u * 64 + lane
    unsigned key[kTinyPerLane];
    unsigned n_nz = 0;
#pragma unroll
    for (int u = 0; u < kTinyPerLane; ++u) {
        const unsigned i = (unsigned)u * 64u + (unsigned)lane;
        key[u] = 0u;
        if (i < n)
            key[u] = score_key(resp[((size_t)(t0 + (int)(i >> 7)) * channels + oc) * kTileRows + (i & 127u)], mode);
        n_nz += (unsigned)__popcll(__ballot(key[u] != 0u));
    }
    ColState st;
    st.tau = 0; st.cut = 0xffffffffu; st.n_eq = 0; st.q = 0; st.tau_lo = 0; st.tau_hi = 0; st.n_nz = n_nz;
    st.n_above = 0; st.side_fill = 0; st.done = 1; st.side_off = 0;
    if (k <= 0) st.tau = 0xffffffffu;  // no key is stronger: nothing survives
    if (k <= 0 || (long long)n_nz <= k) {  // or fewer entries than k: all survive (tau = 0)
        if (lane == 0) cols[col] = st;
        return;
    }
    // 1 <= k < n_nz: the k-th strongest key is non-zero
    unsigned prefix = 0, k_rem = (unsigned)k;
    for (int bit = 31; bit >= 0; --bit) {
        const unsigned want = (prefix >> bit) | 1u;  // the bits from `bit` up of a key with this bit set
        unsigned cnt = 0;
#pragma unroll
        for (int u = 0; u < kTinyPerLane; ++u) cnt += (unsigned)__popcll(__ballot((key[u] >> bit) == want));
        if (cnt >= k_rem) prefix |= 1u << bit;  // the k-th strongest has the bit
        else k_rem -= cnt;                      // it lies below the cnt keys that have it
    }
    const unsigned tau = prefix;
    unsigned n_eq = 0;
#pragma unroll
    for (int u = 0; u < kTinyPerLane; ++u) n_eq += (unsigned)__popcll(__ballot(key[u] == tau));
    const unsigned q = k_rem;  // 1 <= q <= n_eq: the entries equal to tau that survive, those of lowest position
    unsigned cut = 0xffffffffu;
    if (q < n_eq) {
        unsigned left = q;
#pragma unroll
        for (int u = 0; u < kTinyPerLane; ++u) {
            const unsigned long long m = __ballot(key[u] == tau);
            const unsigned c = (unsigned)__popcll(m);
            if (left >= 1u && left <= c) {  // (uniform) the q-th equal key is in this register: the lane of rank `left`
                const unsigned long long hit =
                    __ballot(key[u] == tau && (unsigned)__popcll(m & ((1ull << lane) - 1ull)) + 1u == left);
                cut = (unsigned)u * 64u + (unsigned)(__ffsll((long long)hit) - 1);
                left = 0u;
            } else if (left > c) {
                left -= c;
            }
        }
    }
    if (lane == 0) {
        st.tau = tau;
        st.n_eq = n_eq;
        st.q = q;
        st.cut = cut;
        cols[col] = st;
    }
}

static long long column_positions(const Geom& g) { return (long long)((g.N + kTileRows - 1) / kTileRows) * kTileRows; }

bool topk_small_columns(const Geom& g) {
    return (long long)((g.N + kTileRows - 1) / kTileRows) * kTileRows <= kSmallColumn;
}

// row_keep[w] = the channels' marks for word w (two words per tile) taken together.  A wave takes 64 consecutive
// words; its loads of a plane are one 512-byte piece, eight planes in flight at a time.
__global__ __launch_bounds__(64) void k_combine_marks(int planes, const unsigned long long* __restrict__ row_plane,
                                                      long long plane_words, const Counters* __restrict__ ctr,
                                                      unsigned long long* __restrict__ row_keep) {
    const long long words = 2 * ctr->n_tiles;
    for (long long w = (long long)blockIdx.x * 64 + threadIdx.x; w < words; w += (long long)gridDim.x * 64) {
        unsigned long long m = 0;
        int p = 0;
        for (; p + 8 <= planes; p += 8) {
            unsigned long long x[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) x[j] = row_plane[(size_t)(p + j) * plane_words + w];
#pragma unroll
            for (int j = 0; j < 8; ++j) m |= x[j];
        }
        for (; p < planes; ++p) m |= row_plane[(size_t)p * plane_words + w];
        row_keep[w] = m;
    }
}

hipError_t launch_topk(const Geom& g, int channels, long long k, int mode, int relu, const int* tile_start,
                       const float* resp, ColState* cols, uint2* side, uint2* part, unsigned long long* row_keep,
                       unsigned long long* row_plane, long long* tile_base, long long tiles_cap, Counters* ctr,
                       hipStream_t s) {
    const int ncols = g.batch * channels;
    if (ncols <= 0) return hipSuccess;
    if (column_positions(g) <= kTinyColumn && ncols >= kTinyManyColumns) {
        hipLaunchKernelGGL(k_select_tiny<16>, dim3((unsigned)((ncols + 3) / 4)), dim3(256), 0, s, mode, channels, ncols,
                           tile_start, resp, k, cols);
        return hipGetLastError();
    }
    if (column_positions(g) <= kTinyColumn64 && ncols >= kTinyManyColumns) {
        hipLaunchKernelGGL(k_select_tiny<64>, dim3((unsigned)((ncols + 3) / 4)), dim3(256), 0, s, mode, channels, ncols,
                           tile_start, resp, k, cols);
        return hipGetLastError();
    }
    if (topk_small_columns(g)) {
        hipLaunchKernelGGL(k_select_small, dim3(ncols), dim3(kSmallThreads), 0, s, mode, channels, tile_start, resp, k,
                           cols);
        return hipGetLastError();
    }
    const int groups = g.batch * ((channels + kClassifyWaves - 1) / kClassifyWaves);
    int slices = 2048 / groups;  // (r = 128 layer: 1024 and 4096 workgroups in all measured 2 and 3 us slower)
    if (slices < 1) slices = 1;
    if (slices > kClassifySlicesMax) slices = kClassifySlicesMax;
    const bool marks = row_keep && row_plane && tile_base && k > 0;
    hipLaunchKernelGGL(k_bracket, dim3(ncols), dim3(kBracketThreads), 0, s, mode, channels, tile_start, resp, k, cols);
#define SCNN_CLASSIFY(MODE_, MARKS_)                                                                                 \
    hipLaunchKernelGGL((k_classify<MODE_, MARKS_>), dim3(groups, slices), dim3(kClassifyWaves * 64), 0, s, relu,    \
                       channels, tile_start, resp, cols, side, part, marks ? row_plane : nullptr, 2 * tiles_cap)
    if (mode == SCNN_TOPK_ABS) {
        if (marks) SCNN_CLASSIFY(SCNN_TOPK_ABS, true);
        else SCNN_CLASSIFY(SCNN_TOPK_ABS, false);
    } else {
        if (marks) SCNN_CLASSIFY(SCNN_TOPK_SIGNED, true);
        else SCNN_CLASSIFY(SCNN_TOPK_SIGNED, false);
    }
#undef SCNN_CLASSIFY
    if (marks) {
        long long cb = (2 * tiles_cap + 63) / 64;
        cb = cb < 1 ? 1 : (cb > 2048 ? 2048 : cb);
        hipLaunchKernelGGL(k_combine_marks, dim3((unsigned)cb), dim3(64), 0, s, channels, row_plane, 2 * tiles_cap, ctr,
                           row_keep);
    }
    if (ncols > 256)  // (more columns than compute units: two light workgroups per unit)
        hipLaunchKernelGGL((k_settle<4, 2048u>), dim3(ncols), dim3(kSideThreads), 0, s, mode, relu, channels, k, tile_start,
                           resp, cols, side, part, slices, marks ? row_keep : nullptr, marks ? tile_base : nullptr, ctr);
    else
        hipLaunchKernelGGL((k_settle<20, 12288u>), dim3(ncols), dim3(kSideThreads), 0, s, mode, relu, channels, k,
                           tile_start, resp, cols, side, part, slices, marks ? row_keep : nullptr,
                           marks ? tile_base : nullptr, ctr);
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
    nnz_out[3] = (long long)__hip_atomic_load(&ctr->bracket_failed, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
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
// STREAM: the output row at which every tile starts is known (tile_base, from the rows marked during the
// selection): tiles are dealt out by workgroup index, nothing is published or looked back at, and no tile waits for
// another.  The selection can find, late, that its marks are not to be relied on (ctr->bracket_failed): the kernel
// then works by look-back although it was given tile_base (the choice is uniform over the launch).
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
                                                        int aux_is_cand, const long long* __restrict__ tile_base) {
    const bool STREAM = tile_base != nullptr && ctr->bracket_failed == 0u;
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
    int dealt = (int)blockIdx.x;  // (STREAM) the next tile of this workgroup
    auto next_tile = [&]() -> int {
        if (STREAM) {
            const int t = dealt < n_tiles ? dealt : n_tiles;
            dealt = t + (int)gridDim.x;
            return t;
        }
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
    if (!STREAM && threadIdx.x == 0)
        publish_count(tile_state, tile_x, __popcll(s_mask[0][0]) + __popcll(s_mask[0][1]));
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
                if (!STREAM && tile_y < n_tiles)
                    publish_count(tile_state, tile_y, __popcll(s_mask[slot_y][0]) + __popcll(s_mask[slot_y][1]));
            }
            if (STREAM) {
                if (lane == 0) s_base = tile_base[tile_x];
            } else {
                const int count = __popcll(s_mask[slot_x][0]) + __popcll(s_mask[slot_x][1]);
                const long long base = lookback_published(tile_state, tile_x, count, ctr);
                if (lane == 0) {
                    if (tile_x == n_tiles - 1)
                        __hip_atomic_store(&ctr->n_rows, base + count, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    s_base = base;
                }
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
        nnz_out[3] = (long long)ctr->bracket_failed;
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
// UNI: the wave's tile and sample are made scalars, so that the look-ups of the sample's bounds and of the columns'
// thresholds are scalar loads, once per wave, instead of vector loads per row and channel: fewer instructions, which
// large layers are bound by (128^3 x 4 with 8 channels: 57 -> 48 us), but a chain of dependent scalar loads per row
// group, which small layers, bound by latency, pay for (32^3 network: + 8 us with it everywhere); the host picks by
// the workspace's tile capacity.
constexpr long long kNarrowUniformTiles = 8192;
template <int CMAX, int kNarrowTiles /* tiles per ticket at most: rows per thread = kNarrowTiles / 2 */, bool UNI>
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
            const int tile_v = st * tps + (e >> 7), r = e & (kTileRows - 1);
            const int tile = UNI ? __builtin_amdgcn_readfirstlane(tile_v) : tile_v;
            keep_row[q] = false;
            row_b[q] = 0;
            row_first[q] = -1;
            if ((e >> 7) < tps && tile < n_tiles) {  // (uniform in the wave)
                const int b_v = sample_of_tile(tile_start, g.batch, tile);
                const int b = UNI ? __builtin_amdgcn_readfirstlane(b_v) : b_v;
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
                               long long* nnz_out, long long aux_imm, int aux_is_cand, const long long* tile_base,
                               hipStream_t s) {
    // no more workgroups than can be resident at once (4 per CU by LDS), so that every ticket holder runs; three per
    // CU measured best for the wide kernels (cfg 4: 103 us against 107 with four and 110 with two)
    const long long cus = device_cu_count();
    long long blocks = tiles_cap < 1 ? 1 : (tiles_cap > cus * 3 ? cus * 3 : tiles_cap);
    // Narrow layers: a ticket covers 1, 2, 4 .. NT_ tiles, the fewest that leave at most two tickets per CU (a small
    // layer is bound by the tickets, taken one at a time, and every workgroup launched takes at least one; one per
    // CU and four per CU both measured slower on the paper's networks).
#define SCNN_NARROW_CASE(CMAX_, NT_)                                                                              \
    do {                                                                                                          \
        int tps = 1;                                                                                              \
        while (tps < NT_ && tiles_cap > 512ll * tps) tps *= 2;                                                    \
        long long nb = (tiles_cap + tps - 1) / tps;                                                               \
        nb = nb < 1 ? 1 : (nb > cus * 3 ? cus * 3 : nb);                                                          \
        if (tiles_cap >= kNarrowUniformTiles)                                                                     \
            hipLaunchKernelGGL((k_select_write_narrow<CMAX_, NT_, true>), dim3((unsigned)nb), dim3(256), 0, s, g, \
                               channels, mode, relu, cand_start, tile_start, cand_lin, resp, cols, tile_state,    \
                               ctr, out_coords, out_feats, out_capacity, nnz_out, aux_imm, aux_is_cand, tps);     \
        else                                                                                                      \
            hipLaunchKernelGGL((k_select_write_narrow<CMAX_, NT_, false>), dim3((unsigned)nb), dim3(256), 0, s, g, \
                               channels, mode, relu, cand_start, tile_start, cand_lin, resp, cols, tile_state,    \
                               ctr, out_coords, out_feats, out_capacity, nnz_out, aux_imm, aux_is_cand, tps);     \
    } while (0)
    if (channels <= 4) SCNN_NARROW_CASE(4, 8);
    else if (channels <= 8) SCNN_NARROW_CASE(8, 8);
    else if (channels <= 16) SCNN_NARROW_CASE(16, 8);
    else if (channels <= 32 && !tile_base) SCNN_NARROW_CASE(32, 4);  // (with tile_base: the streaming kernel below)
    else if (channels <= 64) {
        // (streaming: four workgroups per CU; by look-back three measured best, and four cost it 5 %, which only the
        // rare launch that was given tile_base and cannot use it pays)
        if (tile_base) blocks = tiles_cap < 1 ? 1 : (tiles_cap > cus * 4 ? cus * 4 : tiles_cap);
        hipLaunchKernelGGL(k_select_write64, dim3((unsigned)blocks), dim3(256), 0, s, g, channels, mode, relu,
                           cand_start, tile_start, cand_lin, resp, cols, tile_state, ctr, out_coords, out_feats,
                           out_capacity, nnz_out, aux_imm, aux_is_cand, tile_base);
    } else
        hipLaunchKernelGGL(k_select_write, dim3((unsigned)blocks), dim3(256), 0, s, g, channels, mode, relu,
                           cand_start, tile_start, cand_lin, resp, cols, tile_state, ctr, out_coords, out_feats,
                           out_capacity, nnz_out, aux_imm, aux_is_cand);
#undef SCNN_NARROW_CASE
    return hipGetLastError();
}

}  // namespace scnn
