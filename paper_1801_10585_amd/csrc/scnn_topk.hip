// The attention step (Sec. 3.2; Algorithm 1 steps 13, 15-17): per (sample,
// output channel) keep the k strongest non-zero responses, then compact the
// surviving sites into sorted output rows.
//
// Selection = most-significant-digit radix select on an order-preserving 32-bit
// key of the score (three passes of 11 + 11 + 10 bits, histogram in LDS, one
// (column, slice) per workgroup).  It yields the exact k-th largest key tau,
// the number n_eq of entries equal to it and how many of those, q, still fit.
// An entry survives iff  key > tau, or key == tau and it is among the q equal
// entries of lowest lin.  Candidate sites are stored in ascending lin, so that
// rank is a prefix count over the column.
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
__device__ inline void pass_bits(int pass, int& shift, int& bits) {
    shift = pass == 0 ? 21 : (pass == 1 ? 10 : 0);
    bits = pass == 2 ? 10 : 11;
}

// grid = (columns, slices).  Histogram of the current digit over the entries of
// the column that match the prefix found so far.
__global__ __launch_bounds__(256) void k_hist(int pass, int mode, int channels,
                                              const int* __restrict__ tile_start, const float* __restrict__ resp,
                                              const ColState* __restrict__ cols, unsigned* __restrict__ hist) {
    __shared__ unsigned s_hist[kHistBins];
    const int col = blockIdx.x;
    const ColState st = cols[col];
    if (pass > 0 && st.done) return;
    const int b = col / channels, oc = col - b * channels;
    for (int i = threadIdx.x; i < kHistBins; i += 256) s_hist[i] = 0;
    __syncthreads();
    int shift, bits;
    pass_bits(pass, shift, bits);
    const unsigned mask = (1u << bits) - 1u;
    const int t0 = tile_start[b], t1 = tile_start[b + 1];
    const int r = threadIdx.x & (kTileRows - 1);
    for (int tile = t0 + blockIdx.y * 2 + (threadIdx.x >> 7); tile < t1; tile += 2 * gridDim.y) {
        const float v = resp[((size_t)tile * channels + oc) * kTileRows + r];
        const unsigned key = score_key(v, mode);
        if (key == 0u) continue;
        if (pass > 0 && (key >> (shift + bits)) != st.prefix) continue;
        atomicAdd(&s_hist[(key >> shift) & mask], 1u);
    }
    __syncthreads();
    unsigned* gh = hist + (size_t)col * kHistBins;
    for (int i = threadIdx.x; i < kHistBins; i += 256) {
        const unsigned c = s_hist[i];
        if (c) atomicAdd(&gh[i], c);
    }
}

// One block per column: find the bin that holds the k_rem-th strongest entry,
// extend the prefix, clear the histogram for the next pass.
__global__ __launch_bounds__(256) void k_pick(int pass, long long k, ColState* __restrict__ cols,
                                              unsigned* __restrict__ hist, Counters* ctr) {
    __shared__ unsigned s_h[kHistBins];
    __shared__ unsigned s_wave[4];
    const int col = blockIdx.x;
    ColState st;
    if (pass == 0) {
        st.prefix = 0; st.tau = 0; st.k_rem = k; st.n_eq = 0; st.q = 0; st.n_nz = 0; st.done = 0; st.need_tie = 0;
    } else {
        st = cols[col];
        if (st.done) return;  // uniform over the block
    }
    unsigned* gh = hist + (size_t)col * kHistBins;
    unsigned local = 0;  // thread t owns bins [8t, 8t+8); bin 2047 is the strongest
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const unsigned c = gh[threadIdx.x * 8 + i];
        s_h[threadIdx.x * 8 + i] = c;
        gh[threadIdx.x * 8 + i] = 0;
        local += c;
    }
    unsigned total;
    const unsigned excl = block_exclusive_scan_256(local, s_wave, total);
    if (pass == 0) {
        st.n_nz = total;
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
    }
    // Here 1 <= k_rem <= total, so exactly one thread owns the crossing bin.
    const unsigned above_threads = total - excl - local;  // entries in bins owned by higher threads
    const long long k_rem = st.k_rem;
    if ((long long)above_threads < k_rem && k_rem <= (long long)above_threads + (long long)local) {
        unsigned above = above_threads;
        int bin = threadIdx.x * 8 + 7;
        for (; bin > (int)threadIdx.x * 8; --bin) {
            const unsigned c = s_h[bin];
            if (k_rem <= (long long)above + (long long)c) break;
            above += c;
        }
        int shift, bits;
        pass_bits(pass, shift, bits);
        st.prefix = (st.prefix << bits) | (unsigned)bin;
        st.k_rem = k_rem - (long long)above;
        if (pass == 2) {
            st.tau = st.prefix;
            st.n_eq = s_h[bin];
            st.q = (unsigned)st.k_rem;
            st.need_tie = st.q < st.n_eq ? 1 : 0;
            if (st.need_tie) ctr->any_tie = 1;
        }
        cols[col] = st;
    }
}

// Tiles are in ascending (b, lin): the rank of an entry among the entries equal
// to tau is (equal entries in earlier tiles of its column) + (equal entries
// before it in its tile).  These two kernels produce the first term, only for
// columns whose equal entries do not all survive.
__global__ __launch_bounds__(256) void k_tie_count(Geom g, int mode, int channels,
                                                   const int* __restrict__ tile_start,
                                                   const float* __restrict__ resp,
                                                   const ColState* __restrict__ cols,
                                                   unsigned* __restrict__ eqcnt, const Counters* __restrict__ ctr) {
    if (!ctr->any_tie) return;
    const int n_tiles = (int)ctr->n_tiles;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const int b = sample_of_tile(tile_start, g.batch, tile);
        for (int oc = wave; oc < channels; oc += 4) {
            const ColState* st = cols + (size_t)b * channels + oc;
            if (!st->need_tie) continue;
            const unsigned tau = st->tau;
            const float* seg = resp + ((size_t)tile * channels + oc) * kTileRows;
            const unsigned long long m0 = __ballot(score_key(seg[lane], mode) == tau);
            const unsigned long long m1 = __ballot(score_key(seg[64 + lane], mode) == tau);
            if (lane == 0) eqcnt[(size_t)tile * channels + oc] = (unsigned)(__popcll(m0) + __popcll(m1));
        }
    }
}

__global__ __launch_bounds__(256) void k_tie_scan(int channels, const int* __restrict__ tile_start,
                                                  const ColState* __restrict__ cols, unsigned* __restrict__ eqcnt,
                                                  const Counters* __restrict__ ctr) {
    __shared__ unsigned s_wave[4];
    if (!ctr->any_tie) return;
    const int col = blockIdx.x;
    if (!cols[col].need_tie) return;
    const int b = col / channels, oc = col - b * channels;
    const int t0 = tile_start[b], t1 = tile_start[b + 1];
    unsigned carry = 0;
    for (int start = t0; start < t1; start += 256) {
        const int tile = start + threadIdx.x;
        const unsigned v = tile < t1 ? eqcnt[(size_t)tile * channels + oc] : 0u;
        unsigned total;
        const unsigned excl = block_exclusive_scan_256(v, s_wave, total);
        if (tile < t1) eqcnt[(size_t)tile * channels + oc] = carry + excl;
        carry += total;
    }
}

hipError_t launch_topk(const Geom& g, int channels, long long k, int mode, const int* tile_start,
                       const float* resp, ColState* cols, unsigned* hist, unsigned* eqcnt, Counters* ctr,
                       long long tiles_cap, hipStream_t s) {
    const int ncols = g.batch * channels;
    int slices = 2048 / (ncols > 0 ? ncols : 1);
    if (slices < 1) slices = 1;
    if (slices > 64) slices = 64;
    for (int pass = 0; pass < 3; ++pass) {
        hipLaunchKernelGGL(k_hist, dim3(ncols, slices), dim3(256), 0, s, pass, mode, channels, tile_start, resp,
                           cols, hist);
        hipLaunchKernelGGL(k_pick, dim3(ncols), dim3(256), 0, s, pass, k, cols, hist, ctr);
    }
    long long blocks = tiles_cap < 1 ? 1 : (tiles_cap > 2048 ? 2048 : tiles_cap);
    hipLaunchKernelGGL(k_tie_count, dim3((unsigned)blocks), dim3(256), 0, s, g, mode, channels, tile_start, resp,
                       cols, eqcnt, ctr);
    hipLaunchKernelGGL(k_tie_scan, dim3(ncols), dim3(256), 0, s, channels, tile_start, cols, eqcnt, ctr);
    return hipGetLastError();
}

// ------------------------------------------------------------------ keep mask, ReLU, compaction
// WRITE = false: count the surviving rows of every tile.
// WRITE = true : tile_rows holds the scanned row offsets; write the rows.
template <bool WRITE>
__global__ __launch_bounds__(256) void k_select(Geom g, int channels, int mode, int relu,
                                                const int* __restrict__ cand_start,
                                                const int* __restrict__ tile_start,
                                                const unsigned* __restrict__ cand_lin,
                                                const float* __restrict__ resp, const ColState* __restrict__ cols,
                                                const unsigned* __restrict__ eqcnt, unsigned* __restrict__ tile_rows,
                                                const Counters* __restrict__ ctr, int32_t* __restrict__ out_coords,
                                                float* __restrict__ out_feats, long long out_capacity) {
    __shared__ unsigned s_tau[1024];
    __shared__ unsigned s_q[1024];
    __shared__ unsigned char s_tie[1024];
    __shared__ unsigned s_flag[kTileRows];
    __shared__ int s_rank[kTileRows];
    __shared__ int s_wcount[2];
    __shared__ float s_v[WRITE ? kTileRows : 1][65];

    const int n_tiles = (int)ctr->n_tiles;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const unsigned long long lt_mask = (1ull << lane) - 1ull;
    const int n_chunks = (channels + 63) / 64;
    int cur_b = -1;

    for (int tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const int b = sample_of_tile(tile_start, g.batch, tile);
        const int first = cand_start[b] + (tile - tile_start[b]) * kTileRows;
        __syncthreads();
        if (b != cur_b) {
            for (int c = threadIdx.x; c < channels; c += 256) {
                const ColState* st = cols + (size_t)b * channels + c;
                s_tau[c] = st->tau;
                s_q[c] = st->q;
                s_tie[c] = (unsigned char)st->need_tie;
            }
            cur_b = b;
        }
        if (threadIdx.x < kTileRows) s_flag[threadIdx.x] = 0;
        __syncthreads();

        // One wave handles one channel over the tile's 128 rows (two halves, ascending lin).
        auto process = [&](int oc, bool stage, int cc) {
            const float* seg = resp + ((size_t)tile * channels + oc) * kTileRows;
            const unsigned tau = s_tau[oc], q = s_q[oc];
            unsigned running = s_tie[oc] ? eqcnt[(size_t)tile * channels + oc] : 0u;
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                const int r = half * 64 + lane;
                const float v = seg[r];
                const unsigned key = score_key(v, mode);
                const bool eq = (key == tau) && key != 0u;
                const unsigned long long m = __ballot(eq);
                bool keep = key > tau;
                if (eq) keep = (running + (unsigned)__popcll(m & lt_mask)) < q;
                running += (unsigned)__popcll(m);
                if (relu) keep = keep && (v > 0.0f);
                if (keep) s_flag[r] = 1u;
                if (WRITE && stage) s_v[r][oc - cc] = keep ? v : 0.0f;
            }
        };

        if (!WRITE || n_chunks > 1) {
            for (int oc = wave; oc < channels; oc += 4) process(oc, false, 0);
            __syncthreads();
        }
        if (!WRITE) {
            if (threadIdx.x < kTileRows) {
                const unsigned long long m = __ballot(s_flag[threadIdx.x] != 0u);
                if (lane == 0) s_wcount[wave] = __popcll(m);
            }
            __syncthreads();
            if (threadIdx.x == 0) tile_rows[tile] = (unsigned)(s_wcount[0] + s_wcount[1]);
            continue;
        }
        const long long base = tile_rows[tile];
        for (int cc = 0; cc < channels; cc += 64) {
            const int cw = (channels - cc) < 64 ? (channels - cc) : 64;
            for (int oc = cc + wave; oc < cc + cw; oc += 4) process(oc, true, cc);
            __syncthreads();
            if (cc == 0) {
                if (threadIdx.x < kTileRows) {
                    const bool f = s_flag[threadIdx.x] != 0u;
                    const unsigned long long m = __ballot(f);
                    s_rank[threadIdx.x] = __popcll(m & lt_mask);
                    if (lane == 0) s_wcount[wave] = __popcll(m);
                }
                __syncthreads();
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

hipError_t launch_select_write(const Geom& g, int channels, int mode, int relu, const int* cand_start,
                               const int* tile_start, const unsigned* cand_lin, const float* resp,
                               const ColState* cols, const unsigned* eqcnt, unsigned* tile_rows,
                               unsigned* scan_block_sums, long long tiles_cap, Counters* ctr, int32_t* out_coords,
                               float* out_feats, long long out_capacity, long long* n_rows_out, hipStream_t s) {
    long long blocks = tiles_cap < 1 ? 1 : (tiles_cap > 2048 ? 2048 : tiles_cap);
    hipLaunchKernelGGL(k_select<false>, dim3((unsigned)blocks), dim3(256), 0, s, g, channels, mode, relu,
                       cand_start, tile_start, cand_lin, resp, cols, eqcnt, tile_rows, ctr, out_coords, out_feats,
                       out_capacity);
    hipError_t e = launch_exclusive_scan(tile_rows, tiles_cap, 0, &ctr->n_tiles, scan_block_sums, n_rows_out, s);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_select<true>, dim3((unsigned)blocks), dim3(256), 0, s, g, channels, mode, relu,
                       cand_start, tile_start, cand_lin, resp, cols, eqcnt, tile_rows, ctr, out_coords, out_feats,
                       out_capacity);
    return hipGetLastError();
}

}  // namespace scnn
