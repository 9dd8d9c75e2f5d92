// Row-list operators: sparse ReLU, sparse max-pooling (Sec. 3.3), validation.
//
// Pooling in the paper is: rewrite keys (divide the spatial index by the
// stride), sort, reduce each cluster.  Here the sort is replaced by a bitmap
// over the pooled grid: marking every row's pooled site and prefix-counting the
// bitmap yields the output rows already in ascending (b, lin) order; each
// output site then gathers its 2^d children through the occupancy index of the
// input rows and takes the maximum over the entries that are present.  No
// atomics on values, so the result does not depend on scheduling.
#include "scnn_internal.h"

namespace scnn {

// ------------------------------------------------------------------ ReLU
__global__ __launch_bounds__(256) void k_relu_flag(const float* __restrict__ feats, long long rows, int channels,
                                                   unsigned* __restrict__ flags, unsigned* __restrict__ offs) {
    // 16 lanes per row
    const long long gid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const int sub = threadIdx.x & 15;
    const int lane = threadIdx.x & 63;
    for (long long r0 = gid >> 4; r0 < round_up(rows, 16); r0 += ((long long)gridDim.x * blockDim.x) >> 4) {
        bool any = false;
        if (r0 < rows)
            for (int c = sub; c < channels; c += 16) any |= feats[r0 * channels + c] > 0.0f;
        const unsigned long long m = __ballot(any);
        const unsigned seg = (unsigned)((m >> (lane & ~15)) & 0xffffull);
        if (sub == 0 && r0 < rows) {
            flags[r0] = seg ? 1u : 0u;
            offs[r0] = seg ? 1u : 0u;
        }
    }
}

__global__ __launch_bounds__(256) void k_relu_write(Geom g, const int32_t* __restrict__ coords,
                                                    const float* __restrict__ feats, long long rows, int channels,
                                                    const unsigned* __restrict__ flags,
                                                    const unsigned* __restrict__ offs,
                                                    int32_t* __restrict__ out_coords, float* __restrict__ out_feats,
                                                    long long out_capacity) {
    const long long total = rows * channels;
    const int stride = 1 + g.ndim;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (long long)gridDim.x * blockDim.x) {
        const long long r = i / channels;
        const int c = (int)(i - r * channels);
        if (!flags[r]) continue;
        const long long o = offs[r];
        if (o >= out_capacity) continue;
        const float v = feats[i];
        out_feats[o * channels + c] = v > 0.0f ? v : 0.0f;
        if (c == 0)
            for (int j = 0; j < stride; ++j) out_coords[o * stride + j] = coords[r * stride + j];
    }
}

hipError_t launch_relu(const Geom& g, const int32_t* coords, const float* feats, long long rows, int channels,
                       unsigned* flags, unsigned* offs, unsigned* scan_block_sums, int32_t* out_coords,
                       float* out_feats, long long out_capacity, Counters* ctr, hipStream_t s) {
    long long blocks = (rows * 16 + 255) / 256;
    if (blocks < 1) blocks = 1;
    if (blocks > 8192) blocks = 8192;
    hipLaunchKernelGGL(k_relu_flag, dim3((unsigned)blocks), dim3(256), 0, s, feats, rows, channels, flags, offs);
    hipError_t e = launch_exclusive_scan(offs, rows, rows, nullptr, scan_block_sums, &ctr->n_rows, s);
    if (e != hipSuccess) return e;
    blocks = (rows * channels + 255) / 256;
    if (blocks < 1) blocks = 1;
    if (blocks > 16384) blocks = 16384;
    hipLaunchKernelGGL(k_relu_write, dim3((unsigned)blocks), dim3(256), 0, s, g, coords, feats, rows, channels,
                       flags, offs, out_coords, out_feats, out_capacity);
    return hipGetLastError();
}

// ------------------------------------------------------------------ max-pooling
// rows_have_entries != 0: the caller guarantees that every row holds a non-zero entry (skip the check).
__global__ __launch_bounds__(256) void k_pool_mark(Geom g, Geom gp, const int32_t* __restrict__ coords,
                                                   const float* __restrict__ feats, int channels,
                                                   int rows_have_entries, long long n_imm,
                                                   const long long* __restrict__ n_dev,
                                                   unsigned long long* __restrict__ pbits) {
    const long long n = n_dev ? *n_dev : n_imm;
    const int stride = 1 + g.ndim;
    const int lane = threadIdx.x & 63;
    for (long long base = (long long)blockIdx.x * blockDim.x; base < n; base += (long long)gridDim.x * blockDim.x) {
        const long long r = base + threadIdx.x;
        long long key = -1;
        if (r < n) {
            int b, c0, c1, c2;
            load_site(g, coords + r * stride, b, c0, c1, c2);
            bool any = site_in_grid(g, b, c0, c1, c2);
            if (any && !rows_have_entries) {  // a row of zeros holds no entry and creates no output site
                // (stops at the first non-zero value, which an ordinary row has in its first few channels; 16 bytes
                // at a time where the rows allow it)
                any = false;
                const float* row = feats + r * channels;
                if ((channels & 3) == 0 && (((size_t)feats) & 15) == 0) {
                    for (int c = 0; c < channels && !any; c += 4) {
                        const float4 v = *reinterpret_cast<const float4*>(row + c);
                        any = v.x != 0.0f || v.y != 0.0f || v.z != 0.0f || v.w != 0.0f;
                    }
                } else {
                    for (int c = 0; c < channels && !any; ++c) any = row[c] != 0.0f;
                }
            }
            if (any) key = (long long)b * gp.Npad + lin_of(gp, c0 >> 1, c1 >> 1, c2 >> 1);
        }
        // neighbouring rows fall into the same output word: one atomic per run of equal words
        const long long word = key >= 0 ? (key >> 6) : (long long)(-1 - lane);
        unsigned long long bits = key >= 0 ? (1ull << (key & 63)) : 0ull;
        const bool first = wave_or_runs(word, bits);
        if (key >= 0 && first) atomicOr(&pbits[word], bits);
    }
}

// The result counters of a pooling call, written by the thread that knows the number of pooled rows (nnz_out may be
// null: a later launch writes them).  Nothing after this point sets a status bit.
__device__ inline void pool_counters(const Counters* ctr, long long rows, long long* nnz_out, long long aux_imm,
                                     int aux_is_cand, long long out_capacity) {
    if (!nnz_out) return;
    unsigned flags = ctr->flags;
    if (rows > out_capacity) flags |= SCNN_FLAG_OUT_OVERFLOW;
    nnz_out[0] = rows;
    nnz_out[1] = aux_is_cand ? ctr->n_cand : aux_imm;
    nnz_out[2] = (long long)flags;
    nnz_out[3] = (long long)ctr->bracket_failed;
}

__global__ __launch_bounds__(256) void k_pool_emit(const unsigned long long* __restrict__ pbits,
                                                   const unsigned* __restrict__ pprefix, long long n_words,
                                                   long long* __restrict__ pool_key, long long pool_cap,
                                                   const Counters* __restrict__ ctr, long long* __restrict__ nnz_out,
                                                   long long aux_imm, int aux_is_cand, long long out_capacity) {
    if (blockIdx.x == 0 && threadIdx.x == 0)  // (the scan before this launch left the total)
        pool_counters(ctr, ctr->n_pool, nnz_out, aux_imm, aux_is_cand, out_capacity);
    for (long long w = (long long)blockIdx.x * blockDim.x + threadIdx.x; w < n_words;
         w += (long long)gridDim.x * blockDim.x) {
        unsigned long long bits = pbits[w];
        long long o = pprefix[w];
        while (bits) {
            const int bit = __ffsll((long long)bits) - 1;
            bits &= bits - 1;
            if (o < pool_cap) pool_key[o] = w * 64 + bit;
            ++o;
        }
    }
}

// The same for short bitmaps (at most kEmitSmallWords words), without the popcount and scan launches before it: a
// block sums the popcounts of the words before its own and scans its 256 words itself; the block that holds the last
// word also knows the total.
__global__ __launch_bounds__(256) void k_pool_emit_small(const unsigned long long* __restrict__ pbits, int n_words,
                                                         long long* __restrict__ pool_key, long long pool_cap,
                                                         Counters* ctr, long long* __restrict__ nnz_out,
                                                         long long aux_imm, int aux_is_cand, long long out_capacity) {
    __shared__ unsigned s_wave[4];
    const int w0 = blockIdx.x * 256;
    unsigned below = 0;
    for (int i0 = threadIdx.x; i0 < w0; i0 += 256 * 8) {  // eight loads in flight per thread
        unsigned long long x[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) x[u] = i0 + 256 * u < w0 ? pbits[i0 + 256 * u] : 0ull;
#pragma unroll
        for (int u = 0; u < 8; ++u) below += (unsigned)__popcll(x[u]);
    }
    unsigned before_block;
    (void)block_exclusive_scan_256(below, s_wave, before_block);
    const int w = w0 + threadIdx.x;
    unsigned long long bits = w < n_words ? pbits[w] : 0ull;
    unsigned block_total;
    long long o = (long long)before_block + block_exclusive_scan_256((unsigned)__popcll(bits), s_wave, block_total);
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) {
        ctr->n_pool = (long long)before_block + block_total;
        pool_counters(ctr, (long long)before_block + block_total, nnz_out, aux_imm, aux_is_cand, out_capacity);
    }
    while (bits) {
        const int bit = __ffsll((long long)bits) - 1;
        bits &= bits - 1;
        if (o < pool_cap) pool_key[o] = (long long)w * 64 + bit;
        ++o;
    }
}

// Bitmaps of up to kEmitMidWords words, two launches instead of four: the candidate counts of chunks of 256 words, then
// blocks that add up the counts of the chunks before their own (one round of loads) and scan their own 256 words.
__global__ __launch_bounds__(256) void k_pool_count_chunks(const unsigned long long* __restrict__ pbits,
                                                           long long n_words, unsigned* __restrict__ chunk_sums) {
    __shared__ unsigned s_wave[4];
    const long long w = (long long)blockIdx.x * 256 + threadIdx.x;
    unsigned n = w < n_words ? (unsigned)__popcll(pbits[w]) : 0u;
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) n += __shfl_xor(n, d, 64);
    if ((threadIdx.x & 63) == 0) s_wave[threadIdx.x >> 6] = n;
    __syncthreads();
    if (threadIdx.x == 0) chunk_sums[blockIdx.x] = s_wave[0] + s_wave[1] + s_wave[2] + s_wave[3];
}

__global__ __launch_bounds__(256) void k_pool_emit_mid(const unsigned long long* __restrict__ pbits,
                                                       const unsigned* __restrict__ chunk_sums, long long n_words,
                                                       long long* __restrict__ pool_key, long long pool_cap,
                                                       Counters* ctr, long long* __restrict__ nnz_out,
                                                       long long aux_imm, int aux_is_cand, long long out_capacity) {
    __shared__ unsigned s_wave[4];
    const int c = blockIdx.x;
    unsigned below = 0;
    for (int i0 = threadIdx.x; i0 < c; i0 += 256 * 8) {  // eight loads in flight per thread
        unsigned x[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) x[u] = i0 + 256 * u < c ? chunk_sums[i0 + 256 * u] : 0u;
#pragma unroll
        for (int u = 0; u < 8; ++u) below += x[u];
    }
    unsigned before_block;
    (void)block_exclusive_scan_256(below, s_wave, before_block);
    const long long w = (long long)c * 256 + threadIdx.x;
    unsigned long long bits = w < n_words ? pbits[w] : 0ull;
    unsigned block_total;
    long long o = (long long)before_block + block_exclusive_scan_256((unsigned)__popcll(bits), s_wave, block_total);
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) {
        ctr->n_pool = (long long)before_block + block_total;
        pool_counters(ctr, (long long)before_block + block_total, nnz_out, aux_imm, aux_is_cand, out_capacity);
    }
    while (bits) {
        const int bit = __ffsll((long long)bits) - 1;
        bits &= bits - 1;
        if (o < pool_cap) pool_key[o] = w * 64 + bit;
        ++o;
    }
}

__global__ __launch_bounds__(256) void k_pool_gather(Geom g, Geom gp, const unsigned long long* __restrict__ occ,
                                                     const unsigned* __restrict__ occ_prefix, long long n_imm,
                                                     const long long* __restrict__ n_dev,
                                                     const float* __restrict__ feats, int channels,
                                                     const long long* __restrict__ pool_key, long long pool_cap,
                                                     const Counters* __restrict__ ctr,
                                                     int32_t* __restrict__ out_coords, float* __restrict__ out_feats,
                                                     long long out_capacity) {
    const long long n_in = n_dev ? *n_dev : n_imm;
    long long n_out = ctr->n_pool;
    if (n_out > pool_cap) n_out = pool_cap;
    if (n_out > out_capacity) n_out = out_capacity;
    // Rows that allow 16-byte accesses: eight lanes share a pooled site.  Lane j looks up child j (one look-up per
    // child and site, whatever the channel count), the eight row indices go round by shuffles, and the lanes then
    // split the site's groups of four channels.
    if ((channels & 3) == 0 && ((((size_t)feats) | ((size_t)out_feats)) & 15) == 0) {
        const int q = channels >> 2;
        const int sub = threadIdx.x & 7;
        const long long sites_per_pass = (long long)gridDim.x * (blockDim.x / 8);
        for (long long o = (long long)blockIdx.x * (blockDim.x / 8) + (threadIdx.x >> 3); o < n_out;
             o += sites_per_pass) {  // (the eight lanes of a site run the same iterations)
            const long long key = pool_key[o];
            const int b = (int)(key / gp.Npad);
            int p0, p1, p2;
            site_of(gp, key - (long long)b * gp.Npad, p0, p1, p2);
            const int mine = lookup_row(g, occ, occ_prefix, n_in, b, 2 * p0 + (sub >> 2), 2 * p1 + ((sub >> 1) & 1),
                                        2 * p2 + (sub & 1));
            int rows[8];
#pragma unroll
            for (int d = 0; d < 8; ++d) rows[d] = __shfl(mine, d, 8);
            for (int cq = sub; cq < q; cq += 8) {
                const int c = cq * 4;
                float best[4] = {0.0f, 0.0f, 0.0f, 0.0f};
                bool present[4] = {false, false, false, false};
#pragma unroll
                for (int d = 0; d < 8; ++d) {
                    if (rows[d] < 0) continue;
                    const float4 v4 = *reinterpret_cast<const float4*>(feats + (size_t)rows[d] * channels + c);
                    const float v[4] = {v4.x, v4.y, v4.z, v4.w};
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        if (v[j] == 0.0f) continue;
                        best[j] = present[j] ? fmaxf(best[j], v[j]) : v[j];
                        present[j] = true;
                    }
                }
                *reinterpret_cast<float4*>(out_feats + o * channels + c) =
                    make_float4(present[0] ? best[0] : 0.0f, present[1] ? best[1] : 0.0f, present[2] ? best[2] : 0.0f,
                                present[3] ? best[3] : 0.0f);
            }
            if (sub == 0) store_site(gp, out_coords + o * (1 + gp.ndim), b, p0, p1, p2);
        }
        return;
    }
    const long long total = n_out * channels;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (long long)gridDim.x * blockDim.x) {
        const long long o = i / channels;
        const int c = (int)(i - o * channels);
        const long long key = pool_key[o];
        const int b = (int)(key / gp.Npad);
        int p0, p1, p2;
        site_of(gp, key - (long long)b * gp.Npad, p0, p1, p2);
        bool present = false;
        float best = 0.0f;
#pragma unroll
        for (int d = 0; d < 8; ++d) {
            const int row = lookup_row(g, occ, occ_prefix, n_in, b, 2 * p0 + (d >> 2), 2 * p1 + ((d >> 1) & 1),
                                       2 * p2 + (d & 1));
            if (row < 0) continue;
            const float v = feats[(size_t)row * channels + c];
            if (v == 0.0f) continue;
            best = present ? fmaxf(best, v) : v;
            present = true;
        }
        out_feats[i] = present ? best : 0.0f;
        if (c == 0) store_site(gp, out_coords + o * (1 + gp.ndim), b, p0, p1, p2);
    }
}

hipError_t launch_maxpool(const Geom& g, const Geom& gp, const int32_t* coords, const float* feats,
                          long long n_imm, const long long* n_dev, long long n_cap, int channels,
                          int rows_have_entries, unsigned long long* occ, unsigned* occ_prefix, unsigned long long* pbits,
                          unsigned* pprefix, unsigned* scan_block_sums, long long* pool_key, long long pool_cap,
                          int32_t* out_coords, float* out_feats, long long out_capacity, Counters* ctr,
                          long long* nnz_out, long long aux_imm, int aux_is_cand, hipStream_t s) {
    // occ / pbits must be zero on entry
    hipError_t e = launch_index_build(g, coords, n_imm, n_dev, n_cap, occ, occ_prefix, ctr, s);
    if (e != hipSuccess) return e;
    long long blocks = (n_cap + 255) / 256;
    if (blocks < 1) blocks = 1;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(k_pool_mark, dim3((unsigned)blocks), dim3(256), 0, s, g, gp, coords, feats, channels,
                       rows_have_entries, n_imm, n_dev, pbits);
    const long long n_words = (long long)gp.batch * gp.Wps;
    if (n_words <= kEmitSmallWords) {
        hipLaunchKernelGGL(k_pool_emit_small, dim3((unsigned)((n_words + 255) / 256)), dim3(256), 0, s, pbits,
                           (int)n_words, pool_key, pool_cap, ctr, nnz_out, aux_imm, aux_is_cand, out_capacity);
    } else if (n_words <= kEmitMidWords) {  // (scan_block_sums holds at least a counter per 256 words then)
        const unsigned chunks = (unsigned)((n_words + 255) / 256);
        hipLaunchKernelGGL(k_pool_count_chunks, dim3(chunks), dim3(256), 0, s, pbits, n_words, scan_block_sums);
        hipLaunchKernelGGL(k_pool_emit_mid, dim3(chunks), dim3(256), 0, s, pbits, scan_block_sums, n_words, pool_key,
                           pool_cap, ctr, nnz_out, aux_imm, aux_is_cand, out_capacity);
    } else {
        e = launch_popcount(pbits, n_words, pprefix, s);
        if (e != hipSuccess) return e;
        e = launch_exclusive_scan(pprefix, n_words, n_words, nullptr, scan_block_sums, &ctr->n_pool, s);
        if (e != hipSuccess) return e;
        blocks = (n_words + 255) / 256;
        if (blocks > 4096) blocks = 4096;
        hipLaunchKernelGGL(k_pool_emit, dim3((unsigned)blocks), dim3(256), 0, s, pbits, pprefix, n_words, pool_key,
                           pool_cap, ctr, nnz_out, aux_imm, aux_is_cand, out_capacity);
    }
    // (eight lanes per pooled site in the 16-byte form, a thread per value otherwise)
    const bool vec4 = (channels & 3) == 0 && ((((size_t)feats) | ((size_t)out_feats)) & 15) == 0;
    blocks = ((vec4 ? pool_cap * 8 : pool_cap * channels) + 255) / 256;
    if (blocks < 1) blocks = 1;
    if (blocks > 16384) blocks = 16384;
    hipLaunchKernelGGL(k_pool_gather, dim3((unsigned)blocks), dim3(256), 0, s, g, gp, occ, occ_prefix, n_imm, n_dev,
                       feats, channels, pool_key, pool_cap, ctr, out_coords, out_feats, out_capacity);
    return hipGetLastError();
}

// ------------------------------------------------------------------ validation
__global__ __launch_bounds__(256) void k_validate(Geom g, const int32_t* __restrict__ coords, long long rows,
                                                  Counters* ctr) {
    const int stride = 1 + g.ndim;
    for (long long r = (long long)blockIdx.x * blockDim.x + threadIdx.x; r < rows;
         r += (long long)gridDim.x * blockDim.x) {
        int b, c0, c1, c2;
        load_site(g, coords + r * stride, b, c0, c1, c2);
        if (!site_in_grid(g, b, c0, c1, c2)) {
            atomicOr(&ctr->flags, SCNN_FLAG_BAD_COORD);
            continue;
        }
        if (r > 0) {
            int pb, p0, p1, p2;
            load_site(g, coords + (r - 1) * stride, pb, p0, p1, p2);
            if (site_in_grid(g, pb, p0, p1, p2)) {
                const long long key = (long long)b * g.Npad + lin_of(g, c0, c1, c2);
                const long long prev = (long long)pb * g.Npad + lin_of(g, p0, p1, p2);
                if (prev >= key) atomicOr(&ctr->flags, SCNN_FLAG_UNSORTED);
            }
        }
    }
}

hipError_t launch_validate(const Geom& g, const int32_t* coords, long long rows, Counters* ctr, hipStream_t s) {
    long long blocks = (rows + 255) / 256;
    if (blocks < 1) blocks = 1;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(k_validate, dim3((unsigned)blocks), dim3(256), 0, s, g, coords, rows, ctr);
    return hipGetLastError();
}

// ------------------------------------------------------------------ sparseToDense
// dense[b][c][lin] = feats[row(b, lin)][c]; every other element 0.  The fill and the scatter are two launches on
// the same stream.  Rows outside the grid are skipped.
__global__ __launch_bounds__(256) void k_dense_fill(float* __restrict__ dense, size_t n) {
    const size_t n4 = n / 4;  // dense is 16-byte aligned
    float4* d4 = (float4*)dense;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride)
        d4[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (blockIdx.x == 0 && threadIdx.x < (n & 3)) dense[n4 * 4 + threadIdx.x] = 0.f;
}

__global__ __launch_bounds__(256) void k_dense_scatter(Geom g, const int32_t* __restrict__ coords,
                                                       const float* __restrict__ feats, long long rows_cap,
                                                       const long long* __restrict__ rows_dev, int channels,
                                                       float* __restrict__ dense) {
    const int stride = 1 + g.ndim;
    long long rows = rows_dev ? *rows_dev : rows_cap;
    if (rows > rows_cap) rows = rows_cap;
    const long long total = rows * channels;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (long long)gridDim.x * blockDim.x) {
        const long long r = i / channels;
        const int c = (int)(i - r * channels);
        int b, c0, c1, c2;
        load_site(g, coords + r * stride, b, c0, c1, c2);
        if (!site_in_grid(g, b, c0, c1, c2)) continue;
        dense[((size_t)b * channels + c) * (size_t)g.N + (size_t)lin_of(g, c0, c1, c2)] = feats[i];
    }
}

hipError_t launch_to_dense(const Geom& g, const int32_t* coords, const float* feats, long long rows,
                           const long long* rows_dev, int channels, float* dense, hipStream_t s) {
    const size_t n = (size_t)g.batch * channels * (size_t)g.N;
    size_t fb = (n / 4 + 255) / 256;
    if (fb < 1) fb = 1;
    if (fb > 4096) fb = 4096;
    hipLaunchKernelGGL(k_dense_fill, dim3((unsigned)fb), dim3(256), 0, s, dense, n);
    if (rows > 0) {
        long long sb = (rows * channels + 255) / 256;
        if (sb > 8192) sb = 8192;
        hipLaunchKernelGGL(k_dense_scatter, dim3((unsigned)sb), dim3(256), 0, s, g, coords, feats, rows, rows_dev,
                           channels, dense);
    }
    return hipGetLastError();
}

}  // namespace scnn
