// Convolution proper (Algorithm 1, steps 5-9 and 13-14), output-stationary.
//
// The paper scatters every input entry into a dense per-(sample, channel)
// buffer with atomic adds.  Here each candidate output site instead gathers
// its present neighbours: for tap delta the neighbour of p is q = p + delta,
// found through the occupancy bitmap (the inverse of get_update_id).  Sums are
// therefore formed in a fixed order (tap ascending, input channel ascending),
// need no atomics and no r^d value buffer, and are bit-reproducible.
//
// Accumulation is in fp64 with one rounding to fp32 per response: a response is
// a sum of hundreds of signed products that largely cancel, and an fp32 running
// sum leaves an absolute error of a few 1e-6 on the small ones -- more than the
// 1e-6 the layer's results are held to.  On gfx950 the fp64 vector FMA issues at
// the rate of the (unpacked) fp32 one, so the wider sum costs registers only.
//
// Responses are written as tiles of kTileRows candidate sites in a planar
// layout  resp[tile][oc][row]  so that the per-channel selection that follows
// streams contiguous segments.
#include <type_traits>

#include "scnn_internal.h"

namespace scnn {

constexpr int kTapChunk = 32;  // taps whose neighbour rows are staged in LDS at a time
constexpr int kOcBlock = 16;   // output channels accumulated per thread

// Streaming form of the vector kernel, for layers with many more work items than workgroup slots: little shared
// memory and moderate registers, so that many waves per compute unit hide each other's memory latency.  A thread
// walks its taps; per tap it fetches CH input channels with one vector load and takes the weights through scalar
// loads, two channels' worth at a time.  Neighbour rows are looked up per filter line (adjacent sites share one
// pair of bitmap words).
// Work item = (tile, block of 32 output channels); thread = (row, 16 channels).  When the block holds only 16
// channels the second half of the workgroup takes every other tap (partial sums added through LDS, fixed order).
// OCB = 8: layers of at most 8 output channels (the first block of the paper's networks, on its largest grid) keep
// 8 accumulators per thread instead of 16 half-idle ones; on such layers the kernel is bound by FMA issue.
// Runs only when the layer has more than `min_items` work items (a device-side count).
template <int CH /* the largest of 8, 4, 2, 1 that divides C_in and suits the alignment of the values */,
          int OCB /* output channels per thread: 16, or 8 for layers of at most 8 channels (then always split) */>
__global__ __launch_bounds__(256) void k_conv_valu_stream(Geom g, const unsigned long long* __restrict__ occ,
                                                          const unsigned* __restrict__ occ_prefix, long long nnz_in,
                                                          const float* __restrict__ feats, int c_in,
                                                          const double* __restrict__ wp, int c_out, int c_out_pad,
                                                          const float* __restrict__ bias,
                                                          const int* __restrict__ tap_active,
                                                          const unsigned* __restrict__ cand_lin,
                                                          const int* __restrict__ cand_start,
                                                          const int* __restrict__ tile_start,
                                                          const Counters* __restrict__ ctr, long long min_items,
                                                          float* __restrict__ resp) {
    // s_nbr doubles as the buffer of the second half's partial sums (16 doubles per row fit in 33 ints)
    __shared__ __align__(8) int s_nbr[kTileRows][kTapChunk + 2];
    __shared__ int s_site[kTileRows][3];
    static_assert(sizeof(int) * (kTapChunk + 2) >= sizeof(double) * (kOcBlock + 1), "a row of partial sums fits");

    const int n_tiles = (int)ctr->n_tiles;
    const int n_chunks = (c_out_pad + 2 * kOcBlock - 1) / (2 * kOcBlock);
    const long long n_items = (long long)n_tiles * n_chunks;
    if (n_items <= min_items) return;  // the latency-oriented kernel takes small layers
    const int row = threadIdx.x & (kTileRows - 1);
    const int half = __builtin_amdgcn_readfirstlane(threadIdx.x >> 7);  // which 16-channel block of the chunk

    for (long long item = blockIdx.x; item < n_items; item += gridDim.x) {
        const int tile = (int)(item / n_chunks);
        const int chunk = (int)(item - (long long)tile * n_chunks);
        const int b = sample_of_tile(tile_start, g.batch, tile);
        const int first = cand_start[b] + (tile - tile_start[b]) * kTileRows;
        int nrows = cand_start[b + 1] - first;
        if (nrows > kTileRows) nrows = kTileRows;
        const bool split = chunk * 2 * kOcBlock + kOcBlock >= c_out_pad;
        const int oc0 = chunk * 2 * kOcBlock + (split ? 0 : half * kOcBlock);

        __syncthreads();  // previous item's readers of s_site / s_nbr are done
        if (threadIdx.x < kTileRows) {
            int c0 = 0, c1 = 0, c2 = 0;
            if (threadIdx.x < nrows) site_of(g, cand_lin[first + threadIdx.x], c0, c1, c2);
            s_site[threadIdx.x][0] = c0;
            s_site[threadIdx.x][1] = c1;
            s_site[threadIdx.x][2] = c2;
        }

        double acc[OCB];
#pragma unroll
        for (int o = 0; o < OCB; ++o) acc[o] = 0.0;

        for (int tc = 0; tc < g.T; tc += kTapChunk) {
            const int tmax = (g.T - tc) < kTapChunk ? (g.T - tc) : kTapChunk;
            __syncthreads();
            // element i = line segment * 128 + row: the chunk's taps are cut into runs that share (t0, t1); a run's
            // neighbours are adjacent sites and are resolved from one pair of bitmap words
            {
                const int l_first = tc / g.K[2];
                const int n_seg = (tc + tmax - 1) / g.K[2] - l_first + 1;
                for (int i = threadIdx.x; i < kTileRows * n_seg; i += 256) {
                    const int r = i & (kTileRows - 1), l = l_first + (i >> 7);
                    const int ta = tc > l * g.K[2] ? tc : l * g.K[2];
                    const int tb = (tc + tmax) < (l + 1) * g.K[2] ? (tc + tmax) : (l + 1) * g.K[2];
                    const int t0 = l / g.K[1], t1 = l - t0 * g.K[1];
                    int* dst = &s_nbr[r][ta - tc];
                    lookup_line(g, occ, occ_prefix, nnz_in, r < nrows, b, s_site[r][0], s_site[r][1], s_site[r][2], t0,
                                t1, ta - l * g.K[2], tb - ta, tap_active + ta, [&](int k, int n) { dst[k] = n; });
                }
            }
            __syncthreads();
            if (oc0 < c_out_pad && row < nrows) {
                for (int tt = split ? half : 0; tt < tmax; tt += split ? 2 : 1) {
                    const int n = s_nbr[row][tt];
                    if (n < 0) continue;
                    const float* __restrict__ x = feats + (size_t)n * c_in;
                    const double* __restrict__ wt = wp + ((size_t)(tc + tt) * c_in) * c_out_pad + oc0;
                    for (int ic0 = 0; ic0 < c_in; ic0 += CH) {
                        float xv[CH];
                        if constexpr (CH == 8) {
                            const float4 u = *(const float4*)(x + ic0), v = *(const float4*)(x + ic0 + 4);
                            xv[0] = u.x; xv[1] = u.y; xv[2] = u.z; xv[3] = u.w;
                            xv[4] = v.x; xv[5] = v.y; xv[6] = v.z; xv[7] = v.w;
                        } else if constexpr (CH == 4) {
                            const float4 u = *(const float4*)(x + ic0);
                            xv[0] = u.x; xv[1] = u.y; xv[2] = u.z; xv[3] = u.w;
                        } else if constexpr (CH == 2) {
                            const float2 u = *(const float2*)(x + ic0);
                            xv[0] = u.x; xv[1] = u.y;
                        } else {
                            xv[0] = x[ic0];
                        }
                        // two channels' weights (64 scalar registers) in flight at a time: more would spill
#pragma unroll
                        for (int j2 = 0; j2 < CH; j2 += 2) {
                            const double* __restrict__ wr = wt + (size_t)(ic0 + j2) * c_out_pad;
                            double wa[OCB], wb[OCB];
#pragma unroll
                            for (int o = 0; o < OCB; ++o) wa[o] = wr[o];
                            if constexpr (CH > 1) {
#pragma unroll
                                for (int o = 0; o < OCB; ++o) wb[o] = wr[c_out_pad + o];
                            }
                            const double xa = (double)xv[j2];
#pragma unroll
                            for (int o = 0; o < OCB; ++o) acc[o] = fma(xa, wa[o], acc[o]);
                            if constexpr (CH > 1) {
                                const double xb = (double)xv[j2 + 1];
#pragma unroll
                                for (int o = 0; o < OCB; ++o) acc[o] = fma(xb, wb[o], acc[o]);
                            }
                            // keeps the compiler from hoisting the next pair's scalar loads above this point
                            asm volatile("" ::: "memory");
                        }
                    }
                }
            }
        }
        if (split) {  // even taps (first half) + odd taps (second half)
            double* s_acc = reinterpret_cast<double*>(&s_nbr[row][0]);
            __syncthreads();  // the last chunk's neighbour rows have been read
            if (half == 1) {
#pragma unroll
                for (int o = 0; o < OCB; ++o) s_acc[o] = acc[o];
            }
            __syncthreads();
            if (half == 0) {
#pragma unroll
                for (int o = 0; o < OCB; ++o) acc[o] += s_acc[o];
            }
        }
        if (oc0 < c_out_pad && (!split || half == 0)) {
#pragma unroll
            for (int o = 0; o < OCB; ++o) {
                const int oc = oc0 + o;
                if (oc < c_out) {
                    float v = (row < nrows) ? (float)acc[o] : 0.0f;
                    if (bias && v != 0.0f) v += bias[oc];
                    resp[((size_t)tile * c_out + oc) * kTileRows + row] = v;
                }
            }
        }
    }
}

// Response tiles of a layer without input rows (candidate sites cannot exist either; kept for completeness).
__global__ __launch_bounds__(256) void k_conv_valu_empty(int c_out, const Counters* __restrict__ ctr,
                                                         float* __restrict__ resp) {
    const size_t n = (size_t)ctr->n_tiles * c_out * kTileRows;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
        resp[i] = 0.0f;
}

typedef double f64x4 __attribute__((ext_vector_type(4)));

// Latency-oriented form of the vector kernel, for layers with at most `max_items` work items (about one per
// workgroup slot of the chip: the regime of the paper's own narrow networks on small grids).
// Work item = (tile, block of 32 output channels); thread = (row, 16 channels).  When the block has only 16
// channels (C_out <= 16, or the last block), the second half of the workgroup would idle: it then takes every
// other tap of the same 16 channels instead and the two partial sums are added through LDS (even taps + odd taps,
// a fixed order).
// What bounds a small layer is memory latency, not arithmetic, so nothing in the inner loop waits on global memory:
// the neighbour rows of a chunk of taps are looked up per filter line (adjacent sites share one pair of bitmap
// words), and the neighbours' values are gathered into LDS cooperatively (CH channels of TG taps at a time, every
// load independent of every other), together with the group's weights, one round ahead of the multiply-add phase
// that reads both from there.
// With CH >= 4 the multiply-add phase runs on the fp64 matrix cores instead (v_mfma_f64_16x16x4_f64, same fp64
// products and sums): wave w then owns rows 32 w .. 32 w + 31 and all of the chunk's channels, and the results go
// through LDS to the (row, 16 channels) threads that write them.  Reading a (tap, channel)'s 16 weights as an LDS
// broadcast per lane, as the thread-per-row form does, costs the LDS four times the cycles the FMAs take.
template <int CH /* input channels per gather: the largest of 8, 4, 2, 1 that divides C_in */>
__global__ __launch_bounds__(256) void k_conv_valu(Geom g, const unsigned long long* __restrict__ occ,
                                                   const unsigned* __restrict__ occ_prefix, long long nnz_in,
                                                   const float* __restrict__ feats, int c_in,
                                                   const double* __restrict__ wp, int c_out, int c_out_pad,
                                                   const float* __restrict__ bias,
                                                   const int* __restrict__ tap_active,
                                                   const unsigned* __restrict__ cand_lin,
                                                   const int* __restrict__ cand_start,
                                                   const int* __restrict__ tile_start,
                                                   const Counters* __restrict__ ctr, long long max_items,
                                                   float* __restrict__ resp) {
    constexpr int TG = (64 / CH) < kTapChunk ? (64 / CH) : kTapChunk;  // taps per gather
    constexpr int XS = TG * CH + 4;                                     // row stride of the gathered values
    __shared__ int s_nbr[kTileRows][kTapChunk + 1];
    __shared__ int s_site[kTileRows][3];
    __shared__ __align__(16) float s_x[kTileRows][XS];
    __shared__ __align__(16) double s_w[2][TG * CH][kOcBlock];  // the group's weights, per 16-channel block
    // partial sums of the second half when it shares the taps; reuses the gather buffer after the last group
    static_assert(sizeof(float) * XS >= sizeof(double) * (kOcBlock + 1), "gather rows hold a row of partial sums");
    double (*s_acc)[kOcBlock + 1] = reinterpret_cast<double (*)[kOcBlock + 1]>(&s_x[0][0]);

    const int n_tiles = (int)ctr->n_tiles;
    const int n_chunks = (c_out_pad + 2 * kOcBlock - 1) / (2 * kOcBlock);
    const long long n_items = (long long)n_tiles * n_chunks;
    if (n_items > max_items) return;  // the streaming kernel takes large layers
    const int row = threadIdx.x & (kTileRows - 1);
    const int half = __builtin_amdgcn_readfirstlane(threadIdx.x >> 7);  // which 16-channel block of the chunk

    for (long long item = blockIdx.x; item < n_items; item += gridDim.x) {
        const int tile = (int)(item / n_chunks);
        const int chunk = (int)(item - (long long)tile * n_chunks);
        const int b = sample_of_tile(tile_start, g.batch, tile);
        const int first = cand_start[b] + (tile - tile_start[b]) * kTileRows;
        int nrows = cand_start[b + 1] - first;
        if (nrows > kTileRows) nrows = kTileRows;
        // the chunk's second 16-channel block does not exist: both halves work on the first one, taps interleaved
        const bool split = chunk * 2 * kOcBlock + kOcBlock >= c_out_pad;
        const int oc0 = chunk * 2 * kOcBlock + (split ? 0 : half * kOcBlock);

        __syncthreads();  // previous item's readers of the shared arrays are done
        if (threadIdx.x < kTileRows) {
            int c0 = 0, c1 = 0, c2 = 0;
            if (threadIdx.x < nrows) site_of(g, cand_lin[first + threadIdx.x], c0, c1, c2);
            s_site[threadIdx.x][0] = c0;
            s_site[threadIdx.x][1] = c1;
            s_site[threadIdx.x][2] = c2;
        }

        double acc[kOcBlock];
#pragma unroll
        for (int o = 0; o < kOcBlock; ++o) acc[o] = 0.0;
        // matrix-core form (CH >= 4): wave w owns rows 32 w .. 32 w + 31 as two 16-row groups, times the chunk's
        // 16-channel blocks; lane (m, kq) holds output channel m of rows kq, 4 + kq, 8 + kq, 12 + kq of a group
        f64x4 macc[2][2];
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int c = 0; c < 2; ++c) macc[a][c] = f64x4{0.0, 0.0, 0.0, 0.0};
        const int mi = threadIdx.x & 15, kq = (threadIdx.x >> 4) & 3;
        const int wrow = (threadIdx.x >> 6) * 32;  // first row of the wave

        for (int tc = 0; tc < g.T; tc += kTapChunk) {
            const int tmax = (g.T - tc) < kTapChunk ? (g.T - tc) : kTapChunk;
            __syncthreads();
            // ---- neighbour rows of (row, tap): element i = line segment * 128 + row; the chunk's taps are cut into
            //      runs that share (t0, t1), whose neighbours are resolved from one pair of bitmap words
            {
                const int l_first = tc / g.K[2];
                const int n_seg = (tc + tmax - 1) / g.K[2] - l_first + 1;
                for (int i = threadIdx.x; i < kTileRows * n_seg; i += 256) {
                    const int r = i & (kTileRows - 1), l = l_first + (i >> 7);
                    const int ta = tc > l * g.K[2] ? tc : l * g.K[2];
                    const int tb = (tc + tmax) < (l + 1) * g.K[2] ? (tc + tmax) : (l + 1) * g.K[2];
                    const int t0 = l / g.K[1], t1 = l - t0 * g.K[1];
                    int* dst = &s_nbr[r][ta - tc];
                    lookup_line(g, occ, occ_prefix, nnz_in, r < nrows, b, s_site[r][0], s_site[r][1], s_site[r][2], t0,
                                t1, ta - l * g.K[2], tb - ta, tap_active + ta, [&](int k, int n) { dst[k] = n; });
                }
            }
            // ---- rounds = (block of CH input channels) x (group of TG taps).  The global loads of round q + 1 (the
            //      neighbours' values and the group's weights) are in flight while round q multiplies.
            constexpr int GB = (kTileRows * TG) / 256;                   // (row, tap) pairs a thread gathers
            constexpr int WB = (2 * TG * CH * kOcBlock + 255) / 256;     // weights a thread stages
            const int n_tg = (tmax + TG - 1) / TG;
            const int n_rounds = (c_in / CH) * n_tg;
            float xv[GB][CH];
            double wv[WB];
            auto fetch = [&](int q) {
                const int ic0 = (q / n_tg) * CH, tg0 = (q % n_tg) * TG;
                const int tg_n = (tmax - tg0) < TG ? (tmax - tg0) : TG;
#pragma unroll
                for (int m = 0; m < GB; ++m) {
                    const int e = threadIdx.x + m * 256;
                    const int r = e & (kTileRows - 1), tg = e >> 7;
                    const int n = (tg < tg_n) ? s_nbr[r][tg0 + tg] : -1;
                    const float* __restrict__ xp = feats + (size_t)(n < 0 ? 0 : n) * c_in + ic0;
                    if constexpr (CH == 8) {
                        const float4 u = *(const float4*)xp, v = *(const float4*)(xp + 4);
                        xv[m][0] = u.x; xv[m][1] = u.y; xv[m][2] = u.z; xv[m][3] = u.w;
                        xv[m][4] = v.x; xv[m][5] = v.y; xv[m][6] = v.z; xv[m][7] = v.w;
                    } else if constexpr (CH == 4) {
                        const float4 u = *(const float4*)xp;
                        xv[m][0] = u.x; xv[m][1] = u.y; xv[m][2] = u.z; xv[m][3] = u.w;
                    } else if constexpr (CH == 2) {
                        const float2 u = *(const float2*)xp;
                        xv[m][0] = u.x; xv[m][1] = u.y;
                    } else {
                        xv[m][0] = xp[0];
                    }
                    // a site without this neighbour multiplies zeros: the multiply-add phase has no per-row branch
#pragma unroll
                    for (int j = 0; j < CH; ++j) xv[m][j] = n < 0 ? 0.0f : xv[m][j];
                }
                // the group's weights: element e = (hb, tg * CH + j, o) <- w[tap tg][ic0 + j][16 * hb + o of the chunk]
#pragma unroll
                for (int m = 0; m < WB; ++m) {
                    const int e = threadIdx.x + m * 256;
                    const int o = e & (kOcBlock - 1), tj = (e >> 4) % (TG * CH), hb = e / (TG * CH * kOcBlock);
                    const int tg = tj / CH, j = tj - tg * CH;
                    const int oc = chunk * 2 * kOcBlock + hb * kOcBlock + o;
                    const bool ok = e < 2 * TG * CH * kOcBlock && tg < tg_n && oc < c_out_pad;
                    const size_t at = ok ? ((size_t)(tc + tg0 + tg) * c_in + ic0 + j) * c_out_pad + oc : 0;
                    const double v = wp[at];
                    wv[m] = ok ? v : 0.0;
                }
            };
            auto commit = [&]() {
#pragma unroll
                for (int m = 0; m < GB; ++m) {
                    const int e = threadIdx.x + m * 256;
                    const int r = e & (kTileRows - 1), tg = e >> 7;
#pragma unroll
                    for (int j = 0; j < CH; ++j) s_x[r][tg * CH + j] = xv[m][j];
                }
#pragma unroll
                for (int m = 0; m < WB; ++m) {
                    const int e = threadIdx.x + m * 256;
                    if (e < 2 * TG * CH * kOcBlock) (&s_w[0][0][0])[e] = wv[m];
                }
            };
            __syncthreads();  // s_nbr complete
            fetch(0);
            for (int q = 0; q < n_rounds; ++q) {
                const int tg0 = (q % n_tg) * TG;
                const int tg_n = (tmax - tg0) < TG ? (tmax - tg0) : TG;
                __syncthreads();  // the previous round's readers of s_x / s_w are done
                commit();
                __syncthreads();
                if (q + 1 < n_rounds) fetch(q + 1);
                if constexpr (CH >= 4) {
                    // ---- multiply-add on the matrix cores in fp64: per tap and four input channels, the wave's 32
                    //      rows' values (A, 16 x 4 per row group; zeros where a row lacks the neighbour) times the
                    //      weights (B, 4 x 16 per channel block)
                    unsigned live = 0;
#pragma unroll
                    for (int tg = 0; tg < TG; ++tg) {
                        const bool has = tg < tg_n && s_nbr[wrow + (threadIdx.x & 31)][tg0 + tg] >= 0;
                        if (__ballot(has) != 0ull) live |= 1u << tg;
                    }
                    for (int tg = 0; tg < tg_n; ++tg) {
                        if (!((live >> tg) & 1u)) continue;
#pragma unroll
                        for (int jb = 0; jb < CH / 4; ++jb) {
                            const int tj = tg * CH + jb * 4 + kq;
                            const double a0 = (double)s_x[wrow + mi][tj], a1 = (double)s_x[wrow + 16 + mi][tj];
                            const double b0 = s_w[0][tj][mi];
                            macc[0][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b0, macc[0][0], 0, 0, 0);
                            macc[1][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b0, macc[1][0], 0, 0, 0);
                            if (!split) {
                                const double b1 = s_w[1][tj][mi];
                                macc[0][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b1, macc[0][1], 0, 0, 0);
                                macc[1][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b1, macc[1][1], 0, 0, 0);
                            }
                        }
                    }
                    continue;
                }
                // ---- multiply-add: values and weights from LDS (the weights are a broadcast read).  A tap is skipped
                //      when no row of the wave has that neighbour; the weights of input channel j + 1 are read while
                //      channel j multiplies (the fences keep the compiler from sinking the reads to their uses).
                if (oc0 < c_out_pad) {
                    const int hb = split ? 0 : half;
                    unsigned live = 0;
#pragma unroll
                    for (int tg = 0; tg < TG; ++tg) {
                        const bool has = tg < tg_n && s_nbr[row][tg0 + tg] >= 0;
                        if (__ballot(has) != 0ull) live |= 1u << tg;
                    }
                    auto read_w = [&](double (&dst)[kOcBlock], int tj) {
                        const double2* p = reinterpret_cast<const double2*>(&s_w[hb][tj][0]);
#pragma unroll
                        for (int o = 0; o < kOcBlock / 2; ++o) {
                            const double2 v = p[o];
                            dst[2 * o] = v.x;
                            dst[2 * o + 1] = v.y;
                        }
                    };
                    auto mul_add = [&](float x, const double (&wr)[kOcBlock]) {
                        const double xd = (double)x;
#pragma unroll
                        for (int o = 0; o < kOcBlock; ++o) acc[o] = fma(xd, wr[o], acc[o]);
                    };
                    for (int tg = split ? half : 0; tg < tg_n; tg += split ? 2 : 1) {
                        if (!((live >> tg) & 1u)) continue;
                        float xf[CH];
                        if constexpr (CH >= 4) {
#pragma unroll
                            for (int j = 0; j < CH; j += 4) {
                                const float4 u = *reinterpret_cast<const float4*>(&s_x[row][tg * CH + j]);
                                xf[j] = u.x; xf[j + 1] = u.y; xf[j + 2] = u.z; xf[j + 3] = u.w;
                            }
                        } else {
#pragma unroll
                            for (int j = 0; j < CH; ++j) xf[j] = s_x[row][tg * CH + j];
                        }
                        double wa[kOcBlock], wb[kOcBlock];
                        read_w(wa, tg * CH);
#pragma unroll
                        for (int j = 0; j < CH; j += 2) {
                            if (j + 1 < CH) read_w(wb, tg * CH + j + 1);
                            __builtin_amdgcn_sched_barrier(0);
                            mul_add(xf[j], wa);
                            __builtin_amdgcn_sched_barrier(0);
                            if (j + 1 < CH) {
                                if (j + 2 < CH) read_w(wa, tg * CH + j + 2);
                                __builtin_amdgcn_sched_barrier(0);
                                mul_add(xf[j + 1], wb);
                                __builtin_amdgcn_sched_barrier(0);
                            }
                        }
                    }
                }
            }
        }
        if constexpr (CH >= 4) {
            // ---- results to LDS (over the gather buffer), so that a thread can write a row's channels as below
            static_assert(XS >= 2 * kOcBlock + 1, "a gather row holds a row of results");
            __syncthreads();  // the last round's values have been read
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int c = 0; c < 2; ++c)
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        s_x[wrow + a * 16 + 4 * v + kq][c * kOcBlock + mi] = (float)macc[a][c][v];
            __syncthreads();
            if (oc0 < c_out_pad && (!split || half == 0)) {
#pragma unroll
                for (int o = 0; o < kOcBlock; ++o) {
                    const int oc = oc0 + o;
                    if (oc < c_out) {
                        float v = (row < nrows) ? s_x[row][(split ? 0 : half) * kOcBlock + o] : 0.0f;
                        if (bias && v != 0.0f) v += bias[oc];
                        resp[((size_t)tile * c_out + oc) * kTileRows + row] = v;
                    }
                }
            }
            continue;
        }
        if (split) {  // even taps (first half) + odd taps (second half)
            __syncthreads();  // the last group's values have been read
            if (half == 1) {
#pragma unroll
                for (int o = 0; o < kOcBlock; ++o) s_acc[row][o] = acc[o];
            }
            __syncthreads();
            if (half == 0) {
#pragma unroll
                for (int o = 0; o < kOcBlock; ++o) acc[o] += s_acc[row][o];
            }
        }
        if (oc0 < c_out_pad && (!split || half == 0)) {
#pragma unroll
            for (int o = 0; o < kOcBlock; ++o) {
                const int oc = oc0 + o;
                if (oc < c_out) {
                    float v = (row < nrows) ? (float)acc[o] : 0.0f;
                    if (bias && v != 0.0f) v += bias[oc];
                    resp[((size_t)tile * c_out + oc) * kTileRows + row] = v;
                }
            }
        }
    }
}

// The same kernel shape for the smallest layers (at most a few hundred tiles: the deep, pooled layers of the paper's
// networks), where 128-row work items would leave most of the chip idle.  Work item = (quarter of a tile = 32 rows,
// block of 32 output channels).  The four waves of the workgroup share the taps (wave w takes taps w, w + 4, ...);
// A round covers all taps of the chunk for CH input channels, so that a 3^d filter over 24 channels takes three
// rounds.  CH >= 4: a wave multiplies its taps for all 32 rows and channels on the fp64 matrix cores
// (v_mfma_f64_16x16x4_f64) and the four waves' partial sums are added through LDS in the order of the waves.
// CH = 2: the two halves of a wave take the two 16-channel blocks, or, when there is only one, every other input
// channel, with fp64 FMAs; the eight partial sums per output are added through LDS in a fixed order.
template <int CH /* 8, 4 or 2 */>
__global__ __launch_bounds__(256) void k_conv_valu_small(Geom g, const unsigned long long* __restrict__ occ,
                                                         const unsigned* __restrict__ occ_prefix, long long nnz_in,
                                                         const float* __restrict__ feats, int c_in,
                                                         const double* __restrict__ wp, int c_out, int c_out_pad,
                                                         const float* __restrict__ bias,
                                                         const int* __restrict__ tap_active,
                                                         const unsigned* __restrict__ cand_lin,
                                                         const int* __restrict__ cand_start,
                                                         const int* __restrict__ tile_start,
                                                         const Counters* __restrict__ ctr, float* __restrict__ resp) {
    constexpr int R = 32;                    // rows per work item
    constexpr int Q = kTileRows / R;         // work items per tile and channel block
    constexpr int XS = kTapChunk * CH + 4;   // row stride of the gathered values
    constexpr int GB = (R * kTapChunk) / 256;                     // (row, tap) pairs a thread gathers per round
    constexpr int WB = (2 * kTapChunk * CH * kOcBlock) / 256;     // weights a thread stages per round
    __shared__ int s_nbr[R][kTapChunk + 1];
    __shared__ int s_site[R][3];
    __shared__ __align__(16) float s_x[R][XS];
    // the round's weights, per 16-channel block; after the last round the same memory holds the partial sums of
    // the eight (wave, half) pairs
    constexpr int kWElems = 2 * kTapChunk * CH * kOcBlock, kRedElems = 8 * R * (kOcBlock + 1);
    __shared__ __align__(16) double s_wr[kWElems > kRedElems ? kWElems : kRedElems];
    double (*s_w)[kTapChunk * CH][kOcBlock] = reinterpret_cast<double (*)[kTapChunk * CH][kOcBlock]>(&s_wr[0]);
    double (*s_red)[R][kOcBlock + 1] = reinterpret_cast<double (*)[R][kOcBlock + 1]>(&s_wr[0]);

    const int n_tiles = (int)ctr->n_tiles;
    const int n_chunks = (c_out_pad + 2 * kOcBlock - 1) / (2 * kOcBlock);
    const long long n_items = (long long)n_tiles * n_chunks * Q;
    const int row = threadIdx.x & (R - 1);
    const int sl = threadIdx.x >> 5;          // (wave, half of the wave)
    const int lh = sl & 1;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    for (long long item = blockIdx.x; item < n_items; item += gridDim.x) {
        const int quarter = (int)(item % Q);
        const long long tc_item = item / Q;
        const int tile = (int)(tc_item / n_chunks);
        const int chunk = (int)(tc_item - (long long)tile * n_chunks);
        const int b = sample_of_tile(tile_start, g.batch, tile);
        const int first = cand_start[b] + (tile - tile_start[b]) * kTileRows + quarter * R;
        int nrows = cand_start[b + 1] - first;
        if (nrows > R) nrows = R;
        if (nrows < 0) nrows = 0;
        // the chunk's second 16-channel block does not exist: the halves of a wave share the input channels
        const bool split = chunk * 2 * kOcBlock + kOcBlock >= c_out_pad;
        const int hb = split ? 0 : lh;

        double acc[kOcBlock];
#pragma unroll
        for (int o = 0; o < kOcBlock; ++o) acc[o] = 0.0;
        // matrix-core form (CH >= 4): [16-row group][16-channel block]; lane (m, kq) holds output channel m of rows
        // kq, 4 + kq, 8 + kq, 12 + kq (the fp64 instruction's result layout)
        f64x4 macc[2][2];
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int c = 0; c < 2; ++c) macc[a][c] = f64x4{0.0, 0.0, 0.0, 0.0};
        const int mi = threadIdx.x & 15, kq = (threadIdx.x >> 4) & 3;

        __syncthreads();  // previous item's readers of the shared arrays are done
        if (nrows > 0) {  // (uniform) a quarter without rows only writes its zeros
            if (threadIdx.x < R) {
                int c0 = 0, c1 = 0, c2 = 0;
                if (threadIdx.x < nrows) site_of(g, cand_lin[first + threadIdx.x], c0, c1, c2);
                s_site[threadIdx.x][0] = c0;
                s_site[threadIdx.x][1] = c1;
                s_site[threadIdx.x][2] = c2;
            }
            for (int tc = 0; tc < g.T; tc += kTapChunk) {
                const int tmax = (g.T - tc) < kTapChunk ? (g.T - tc) : kTapChunk;
                const int n_rounds = c_in / CH;
                float xv[GB][CH];
                double wv[WB];
                // the round's weights: element e = (block hb, tap tg, channel j, o) <- w[tc + tg][ic0 + j][16 hb + o]
                auto fetch_w = [&](int q) {
                    const int ic0 = q * CH;
#pragma unroll
                    for (int m = 0; m < WB; ++m) {
                        const int e = threadIdx.x + m * 256;
                        const int o = e & (kOcBlock - 1), tj = (e >> 4) % (kTapChunk * CH);
                        const int hbw = e / (kTapChunk * CH * kOcBlock);
                        const int tg = tj / CH, j = tj - tg * CH;
                        const int oc = chunk * 2 * kOcBlock + hbw * kOcBlock + o;
                        const bool ok = tg < tmax && oc < c_out_pad;
                        const size_t at = ok ? ((size_t)(tc + tg) * c_in + ic0 + j) * c_out_pad + oc : 0;
                        const double v = wp[at];
                        wv[m] = ok ? v : 0.0;
                    }
                };
                // the neighbours' values; a site without the neighbour multiplies zeros
                auto fetch_x = [&](int q) {
                    const int ic0 = q * CH;
#pragma unroll
                    for (int m = 0; m < GB; ++m) {
                        const int e = threadIdx.x + m * 256;
                        const int r = e & (R - 1), tg = e >> 5;
                        const int n = (tg < tmax) ? s_nbr[r][tg] : -1;
                        const float* __restrict__ xp = feats + (size_t)(n < 0 ? 0 : n) * c_in + ic0;
                        if constexpr (CH == 8) {
                            const float4 u = *(const float4*)xp, v = *(const float4*)(xp + 4);
                            xv[m][0] = u.x; xv[m][1] = u.y; xv[m][2] = u.z; xv[m][3] = u.w;
                            xv[m][4] = v.x; xv[m][5] = v.y; xv[m][6] = v.z; xv[m][7] = v.w;
                        } else if constexpr (CH == 4) {
                            const float4 u = *(const float4*)xp;
                            xv[m][0] = u.x; xv[m][1] = u.y; xv[m][2] = u.z; xv[m][3] = u.w;
                        } else {
                            const float2 u = *(const float2*)xp;
                            xv[m][0] = u.x; xv[m][1] = u.y;
                        }
#pragma unroll
                        for (int j = 0; j < CH; ++j) xv[m][j] = n < 0 ? 0.0f : xv[m][j];
                    }
                };
                auto commit = [&]() {
#pragma unroll
                    for (int m = 0; m < GB; ++m) {
                        const int e = threadIdx.x + m * 256;
                        const int r = e & (R - 1), tg = e >> 5;
#pragma unroll
                        for (int j = 0; j < CH; ++j) s_x[r][tg * CH + j] = xv[m][j];
                    }
#pragma unroll
                    for (int m = 0; m < WB; ++m) (&s_w[0][0][0])[threadIdx.x + m * 256] = wv[m];
                };
                fetch_w(0);  // does not depend on the neighbours: in flight during the look-ups
                __syncthreads();  // s_site written; the previous chunk's readers of s_nbr are done
                {
                    const int l_first = tc / g.K[2];
                    const int n_seg = (tc + tmax - 1) / g.K[2] - l_first + 1;
                    for (int i = threadIdx.x; i < R * n_seg; i += 256) {
                        const int r = i & (R - 1), l = l_first + (i >> 5);
                        const int ta = tc > l * g.K[2] ? tc : l * g.K[2];
                        const int tb = (tc + tmax) < (l + 1) * g.K[2] ? (tc + tmax) : (l + 1) * g.K[2];
                        const int t0 = l / g.K[1], t1 = l - t0 * g.K[1];
                        int* dst = &s_nbr[r][ta - tc];
                        lookup_line(g, occ, occ_prefix, nnz_in, r < nrows, b, s_site[r][0], s_site[r][1], s_site[r][2],
                                    t0, t1, ta - l * g.K[2], tb - ta, tap_active + ta,
                                    [&](int k, int n) { dst[k] = n; });
                    }
                }
                __syncthreads();  // s_nbr complete
                fetch_x(0);
                // taps of the chunk that some row of this wave has
                unsigned live = 0;
                for (int tg = wave; tg < tmax; tg += 4)
                    if (__ballot(s_nbr[row][tg] >= 0) != 0ull) live |= 1u << tg;
                for (int q = 0; q < n_rounds; ++q) {
                    __syncthreads();  // the previous round's readers of s_x / s_w are done
                    commit();
                    __syncthreads();
                    if (q + 1 < n_rounds) {
                        fetch_w(q + 1);
                        fetch_x(q + 1);
                    }
                    if constexpr (CH >= 4) {
                        // ---- multiply-add on the matrix cores in fp64: per tap and four input channels, the 32
                        //      rows' values (A, 16 x 4 per row group; zeros where a row lacks the neighbour) times
                        //      the weights (B, 4 x 16 per channel block).  Two 8-byte operand reads feed 1024
                        //      multiply-adds, where the vector form reads 128 bytes of weights per lane for 16.
                        for (int tg = wave; tg < tmax; tg += 4) {
                            if (!((live >> tg) & 1u)) continue;
#pragma unroll
                            for (int jb = 0; jb < CH / 4; ++jb) {
                                const int tj = tg * CH + jb * 4 + kq;
                                const double a0 = (double)s_x[mi][tj], a1 = (double)s_x[16 + mi][tj];
                                const double b0 = s_w[0][tj][mi];
                                macc[0][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b0, macc[0][0], 0, 0, 0);
                                macc[1][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b0, macc[1][0], 0, 0, 0);
                                if (!split) {
                                    const double b1 = s_w[1][tj][mi];
                                    macc[0][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b1, macc[0][1], 0, 0, 0);
                                    macc[1][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b1, macc[1][1], 0, 0, 0);
                                }
                            }
                        }
                        continue;
                    }
                    // ---- multiply-add, weights of the next input channel read while this one multiplies
                    auto read_w = [&](double (&dst)[kOcBlock], int tj) {
                        const double2* p = reinterpret_cast<const double2*>(&s_w[hb][tj][0]);
#pragma unroll
                        for (int o = 0; o < kOcBlock / 2; ++o) {
                            const double2 v = p[o];
                            dst[2 * o] = v.x;
                            dst[2 * o + 1] = v.y;
                        }
                    };
                    auto mul_add = [&](float x, const double (&wr)[kOcBlock]) {
                        const double xd = (double)x;
#pragma unroll
                        for (int o = 0; o < kOcBlock; ++o) acc[o] = fma(xd, wr[o], acc[o]);
                    };
                    // channel of step i: every channel, or every other one starting at this half's
                    const int jmul = split ? 2 : 1, jadd = split ? lh : 0;
                    const int n_steps = split ? CH / 2 : CH;
                    for (int tg = wave; tg < tmax; tg += 4) {
                        if (!((live >> tg) & 1u)) continue;
                        double wa[kOcBlock], wb[kOcBlock];
                        const float* xr = &s_x[row][tg * CH + jadd];
                        read_w(wa, tg * CH + jadd);
                        for (int i = 0; i < n_steps; i += 2) {
                            const float xa = xr[i * jmul];
                            float xb = 0.0f;
                            if (i + 1 < n_steps) {
                                xb = xr[(i + 1) * jmul];
                                read_w(wb, tg * CH + (i + 1) * jmul + jadd);
                            }
                            __builtin_amdgcn_sched_barrier(0);
                            mul_add(xa, wa);
                            __builtin_amdgcn_sched_barrier(0);
                            if (i + 1 < n_steps) {
                                if (i + 2 < n_steps) read_w(wa, tg * CH + (i + 2) * jmul + jadd);
                                __builtin_amdgcn_sched_barrier(0);
                                mul_add(xb, wb);
                                __builtin_amdgcn_sched_barrier(0);
                            }
                        }
                    }
                }
            }
        }
        __syncthreads();  // the last round's weights have been read
        if constexpr (CH >= 4) {
            // ---- the four waves' partial sums (one per tap slice), added in the order of the waves
            double (*s_rm)[R][2 * kOcBlock + 1] = reinterpret_cast<double (*)[R][2 * kOcBlock + 1]>(&s_wr[0]);
            static_assert(4 * R * (2 * kOcBlock + 1) <= kRedElems, "the partial sums fit");
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int c = 0; c < 2; ++c)
#pragma unroll
                    for (int v = 0; v < 4; ++v) s_rm[wave][a * 16 + 4 * v + kq][c * kOcBlock + mi] = macc[a][c][v];
            __syncthreads();
            const int per = split ? 2 : 4;  // channels per thread: 16 or 32 channels over 8 thread groups
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (i >= per) break;
                const int c = sl * per + i;  // channel within the chunk
                const int oc = chunk * 2 * kOcBlock + c;
                if (oc >= c_out) continue;
                double sum = 0.0;
#pragma unroll
                for (int k = 0; k < 4; ++k) sum += s_rm[k][row][c];
                float v = (row < nrows) ? (float)sum : 0.0f;
                if (bias && v != 0.0f) v += bias[oc];
                resp[((size_t)tile * c_out + oc) * kTileRows + quarter * R + row] = v;
            }
            continue;
        }
        // ---- the eight partial sums of an output, added in a fixed order (wave 0 .. 3, first half then second)
#pragma unroll
        for (int o = 0; o < kOcBlock; ++o) s_red[sl][row][o] = acc[o];
        __syncthreads();
        {
            const int per = split ? 2 : 4;  // channels per thread: 16 or 32 channels over 8 thread groups
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (i >= per) break;
                const int c = sl * per + i;               // channel within the chunk
                const int hbo = c >> 4, o = c & (kOcBlock - 1);
                const int oc = chunk * 2 * kOcBlock + c;
                if (oc >= c_out) continue;
                double sum = 0.0;
                if (split) {
#pragma unroll
                    for (int k = 0; k < 8; ++k) sum += s_red[k][row][o];
                } else {
#pragma unroll
                    for (int k = 0; k < 4; ++k) sum += s_red[2 * k + hbo][row][o];
                }
                float v = (row < nrows) ? (float)sum : 0.0f;
                if (bias && v != 0.0f) v += bias[oc];
                resp[((size_t)tile * c_out + oc) * kTileRows + quarter * R + row] = v;
            }
        }
    }
}

// Workgroups of the streaming kernel.  About six are resident per CU; a grid of 8 per CU ran a third of them in a
// second, badly filled round (128^3 stack 2.05 ms, paper runtime shape r = 256: convolution 155 us), 6 per CU fits
// exactly (2.02 ms, 137 us), and 32 per CU, about one work item per workgroup on these layers, balances best
// (1.99 ms, 123 us; 64 and 128 per CU the same).
constexpr int kStreamBlocks = 256 * 32;

// Layers with at most this many work items run the latency-oriented kernel, larger ones the streaming kernel.
constexpr long long kValuLatencyItems = 1024;
// Layers whose workspace holds more than this many work items run the streaming kernel alone.
constexpr long long kValuStreamOnlyItems = 8 * kValuLatencyItems;
// Layers whose workspace holds at most this many work items (a bound the host knows) run the 32-row form.
constexpr long long kValuSmallItems = 256;

hipError_t launch_conv_valu(const Geom& g, const unsigned long long* occ, const unsigned* occ_prefix,
                            long long nnz_in, const float* feats, int c_in, const double* wp, int c_out,
                            int c_out_pad, const float* bias, const int* tap_active, const unsigned* cand_lin,
                            const int* cand_start, const int* tile_start, const Counters* ctr, long long tiles_cap,
                            float* resp, hipStream_t s) {
    if (nnz_in <= 0) {  // no input row: every response tile is zero (the gather would have no row to point at)
        hipLaunchKernelGGL(k_conv_valu_empty, dim3(256 * 8), dim3(256), 0, s, c_out, ctr, resp);
        return hipGetLastError();
    }
    // Which kernel runs is decided by the number of work items, which only the device knows.  The host knows an
    // upper bound (tiles_cap): when that is small the latency-oriented kernel is launched alone; otherwise both
    // are launched and the one whose regime it is not returns at once (a few microseconds).
    // Vector loads of CH channels need the row start aligned to them.
    const int align_ch = (int)((((uintptr_t)feats) & 15) == 0 ? 8 : ((((uintptr_t)feats) & 7) == 0 ? 2 : 1));
    int ch = 1;
    if (c_in % 8 == 0 && align_ch >= 8) ch = 8;
    else if (c_in % 4 == 0 && align_ch >= 8) ch = 4;
    else if (c_in % 2 == 0 && align_ch >= 2) ch = 2;
    const int n_chunks = (c_out_pad + 2 * kOcBlock - 1) / (2 * kOcBlock);
    // Far above the latency kernel's regime only the streaming kernel is launched (it takes any number of items; a
    // layer whose workspace is that much larger than its data runs slower on it, a large layer saves a launch).
    const bool stream_only = tiles_cap * n_chunks > kValuStreamOnlyItems;
    const bool both = !stream_only && tiles_cap * n_chunks > kValuLatencyItems;
    if (tiles_cap * n_chunks <= kValuSmallItems && ch >= 2) {  // cannot hold more than a few hundred tiles
        const int blocks = (int)(tiles_cap * n_chunks * (kTileRows / 32));
#define SCNN_VALU_SMALL(CH_)                                                                                         \
    hipLaunchKernelGGL(k_conv_valu_small<CH_>, dim3(blocks), dim3(256), 0, s, g, occ, occ_prefix, nnz_in, feats,     \
                       c_in, wp, c_out, c_out_pad, bias, tap_active, cand_lin, cand_start, tile_start, ctr, resp)
        if (ch == 8) SCNN_VALU_SMALL(8);
        else if (ch == 4) SCNN_VALU_SMALL(4);
        else SCNN_VALU_SMALL(2);
#undef SCNN_VALU_SMALL
        return hipGetLastError();
    }
#define SCNN_VALU_CASE(CH_)                                                                                          \
    do {                                                                                                             \
        const long long stream_min = stream_only ? -1 : kValuLatencyItems;                                           \
        if ((both || stream_only) && c_out <= 8)                                                                     \
            hipLaunchKernelGGL((k_conv_valu_stream<CH_, 8>), dim3(kStreamBlocks), dim3(256), 0, s, g, occ,           \
                               occ_prefix, nnz_in, feats, c_in, wp, c_out, c_out_pad, bias, tap_active, cand_lin,    \
                               cand_start, tile_start, ctr, stream_min, resp);                                       \
        else if (both || stream_only)                                                                                \
            hipLaunchKernelGGL((k_conv_valu_stream<CH_, 16>), dim3(kStreamBlocks), dim3(256), 0, s, g, occ,          \
                               occ_prefix, nnz_in, feats, c_in, wp, c_out, c_out_pad, bias, tap_active, cand_lin,    \
                               cand_start, tile_start, ctr, stream_min, resp);                                       \
        if (!stream_only)                                                                                            \
            hipLaunchKernelGGL(k_conv_valu<CH_>, dim3(256 * 8), dim3(256), 0, s, g, occ, occ_prefix, nnz_in, feats,  \
                               c_in, wp, c_out, c_out_pad, bias, tap_active, cand_lin, cand_start, tile_start, ctr,  \
                               kValuLatencyItems, resp);                                                             \
    } while (0)
    if (ch == 8) SCNN_VALU_CASE(8);
    else if (ch == 4) SCNN_VALU_CASE(4);
    else if (ch == 2) SCNN_VALU_CASE(2);
    else SCNN_VALU_CASE(1);
#undef SCNN_VALU_CASE
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Matrix-core path for wide channels (C_in a multiple of 32, C_out a multiple
// of 16 up to 64): the gathered neighbour block of one tap really is a dense
// [pairs x C_in] . [C_in x C_out] contraction.
//
// Only about a third of a surface candidate's taps have a neighbour, and which
// ones varies from site to site, so zero-padding absent neighbours would waste
// most of the matrix cores.  Instead, per tile of 128 candidate sites and per
// tap, the present (output row, input row) pairs are packed into blocks of 16
// (k_pair_build, a light kernel that runs at high occupancy and leaves the
// lists in global memory); k_conv_mfma then runs one fp32 MFMA chain per block
// and per 32 input channels and adds the 16 x 16 results to the tile's
// accumulators in LDS.  Those accumulators are fp64 (native LDS ds_add_f64):
// the fp32 matrix cores only ever sum 32 products of a single tap, the long
// cancelling sum over channels and taps is carried in double and rounded to
// fp32 once.
//
// A wave multiplies its blocks against a whole filter tap (all C_out channels):
// an input row is fetched once per pair and a tap's weights once per round of
// up to three blocks, which keeps the L1 traffic well below what the matrix
// cores could consume.  Waves of a workgroup share the tile's accumulators
// through the LDS atomic, so the order of the fp64 additions is not fixed.
// ---------------------------------------------------------------------------
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr unsigned kPadPair = (unsigned)kTileRows << kPairRowShift;  // list padding: dummy accumulator row, input row 0
constexpr int kStageBlocks = 208;                 // 16-pair blocks staged in LDS at a time by the contraction

// Pair lists of all tiles live in one global array of 16-entry blocks; a tile's blocks are contiguous, in
// ascending (tap, output row) order.  tile_hdr[tile] = {first block, block count};
// block_tap[block] = tap | (index of the block within its tap) << 8.
// A tile's space is reserved in closed form, at most ceil(rows / 16) blocks per active tap, so a tile starts at
// (active taps) * (16-row groups of all earlier tiles); unused blocks of a reservation are simply never read.
// One wave builds one tile (lanes = output rows lane and lane + 64) and walks the taps in order, so that it needs
// neither barriers nor a scan; the taps are looked up kPairTapGroup at a time to overlap their loads.
constexpr int kPairTapGroup = 4;
__global__ __launch_bounds__(256) void k_pair_build(Geom g, const unsigned long long* __restrict__ occ,
                                                    const unsigned* __restrict__ occ_prefix, long long nnz_in,
                                                    const int* __restrict__ tap_active,
                                                    const int* __restrict__ tap_coord,
                                                    const unsigned* __restrict__ cand_lin,
                                                    const int* __restrict__ cand_start,
                                                    const int* __restrict__ tile_start,
                                                    const int* __restrict__ rows16_start, Counters* ctr,
                                                    unsigned* __restrict__ pairs, unsigned short* __restrict__ block_tap,
                                                    uint2* __restrict__ tile_hdr, long long block_cap,
                                                    unsigned short* __restrict__ tap_first) {
    constexpr int G = kPairTapGroup;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const unsigned long long lt_mask = (1ull << lane) - 1ull;
    const int n_tiles = (int)ctr->n_tiles;
    int active = 0;  // taps with a non-zero weight
    for (int t0 = 0; t0 < g.T; t0 += 64)
        active += __popcll(__ballot(t0 + lane < g.T && tap_active[t0 + lane < g.T ? t0 + lane : 0] != 0));

    const int waves = (int)gridDim.x * 4;
    for (int tile = (int)blockIdx.x * 4 + wave; tile < n_tiles; tile += waves) {
        const int b = sample_of_tile(tile_start, g.batch, tile);
        const int lt = tile - tile_start[b];
        const int first = cand_start[b] + lt * kTileRows;
        int nrows = cand_start[b + 1] - first;
        if (nrows > kTileRows) nrows = kTileRows;
        int sc[2][3];  // sites of rows lane and lane + 64
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            sc[h][0] = sc[h][1] = sc[h][2] = 0;
            if (h * 64 + lane < nrows) site_of(g, cand_lin[first + h * 64 + lane], sc[h][0], sc[h][1], sc[h][2]);
        }
        const long long tile_base = (long long)active * (rows16_start[b] + lt * (kTileRows / 16));
        if (tile_base + (long long)active * ((nrows + 15) >> 4) > block_cap) {
            // cannot happen with the documented workspace size
            if (lane == 0) {
                atomicOr(&ctr->flags, SCNN_FLAG_CAND_OVERFLOW);
                tile_hdr[tile] = make_uint2(0u, 0u);
            }
            if (tap_first)
                for (int t = lane; t <= g.T; t += 64) tap_first[(size_t)tile * (g.T + 1) + t] = 0;
            continue;
        }
        unsigned blk = (unsigned)tile_base;  // next free block
        // Taps are walked in order as segments of up to G taps of one filter line (t0, t1): the neighbours of a
        // segment are adjacent sites, resolved from one pair of bitmap words per row.  Two segments per step keep
        // sixteen loads in flight per lane.
        const int n_sub = (g.K[2] + G - 1) / G;
        const int n_seg = g.K[0] * g.K[1] * n_sub;
        for (int sg0 = 0; sg0 < n_seg; sg0 += 2) {
            unsigned nbr[2][G][2];
            int seg_tap[2], seg_cnt[2];
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int sg = sg0 + u < n_seg ? sg0 + u : n_seg - 1;
                const int line = sg / n_sub, t2_lo = (sg - line * n_sub) * G;
                const int t0l = line / g.K[1], t1l = line - t0l * g.K[1];
                int cnt = g.K[2] - t2_lo;
                if (cnt > G) cnt = G;
                if (sg0 + u >= n_seg) cnt = 0;
                seg_tap[u] = line * g.K[2] + t2_lo;
                seg_cnt[u] = cnt;
#pragma unroll
                for (int h = 0; h < 2; ++h) {
#pragma unroll
                    for (int k = 0; k < G; ++k) nbr[u][k][h] = 0xffffffffu;
                    lookup_line(g, occ, occ_prefix, nnz_in, cnt > 0 && h * 64 + lane < nrows, b, sc[h][0], sc[h][1],
                                sc[h][2], t0l, t1l, t2_lo, cnt, tap_active + seg_tap[u],
                                [&](int k, int n) { nbr[u][k][h] = (unsigned)n; });
                }
            }
            // ---- pack: each tap's present pairs in ascending output row, padded to whole blocks of 16 with
            //      entries that point at the dummy accumulator row
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int m = 0; m < G; ++m) {
                    if (m >= seg_cnt[u]) continue;
                    const int t = seg_tap[u] + m;
                    const unsigned long long m0 = __ballot(nbr[u][m][0] != 0xffffffffu),
                                             m1 = __ballot(nbr[u][m][1] != 0xffffffffu);
                    const int c0 = __popcll(m0), cnt = c0 + __popcll(m1);
                    const int nblk = (cnt + 15) >> 4;
                    unsigned* pl = pairs + (size_t)blk * 16;
                    if (nbr[u][m][0] != 0xffffffffu)
                        pl[__popcll(m0 & lt_mask)] = ((unsigned)lane << kPairRowShift) | nbr[u][m][0];
                    if (nbr[u][m][1] != 0xffffffffu)
                        pl[c0 + __popcll(m1 & lt_mask)] = ((unsigned)(64 + lane) << kPairRowShift) | nbr[u][m][1];
                    if (lane < 16 && cnt + lane < nblk * 16) pl[cnt + lane] = kPadPair;
                    if (lane < nblk) block_tap[blk + lane] = (unsigned short)(t | (lane << 8));
                    // optional: where each tap's blocks start within the tile (entry T = the tile's block count)
                    if (tap_first && lane == 0) tap_first[(size_t)tile * (g.T + 1) + t] = (unsigned short)(blk - (unsigned)tile_base);
                    blk += (unsigned)nblk;
                }
        }
        if (lane == 0) {
            tile_hdr[tile] = make_uint2((unsigned)tile_base, blk - (unsigned)tile_base);
            if (tap_first) tap_first[(size_t)tile * (g.T + 1) + g.T] = (unsigned short)(blk - (unsigned)tile_base);
        }
    }
}

hipError_t launch_pair_build(const Geom& g, const unsigned long long* occ, const unsigned* occ_prefix,
                             long long nnz_in, const int* tap_active, const int* tap_coord,
                             const unsigned* cand_lin, const int* cand_start, const int* tile_start,
                             const int* rows16_start, Counters* ctr, unsigned* pairs, unsigned short* block_tap,
                             uint2* tile_hdr, long long block_cap, long long tiles_cap, unsigned short* tap_first,
                             hipStream_t s) {
    long long blocks = (tiles_cap + 3) / 4;  // one wave per tile
    if (blocks < 1) blocks = 1;
    if (blocks > 256 * 8) blocks = 256 * 8;
    hipLaunchKernelGGL(k_pair_build, dim3((unsigned)blocks), dim3(256), 0, s, g, occ, occ_prefix, nnz_in, tap_active,
                       tap_coord, cand_lin, cand_start, tile_start, rows16_start, ctr, pairs, block_tap, tile_hdr,
                       block_cap, tap_first);
    return hipGetLastError();
}

constexpr int kConvWaves = 4;  // waves per workgroup of the contraction kernel

__host__ __device__ inline size_t conv_mfma_lds_bytes(int c_out) {
    return (size_t)(kTileRows + 1) * (c_out + 1) * sizeof(double)   // accumulators + one dummy row
           + (size_t)kStageBlocks * 16 * sizeof(unsigned)            // staged pair blocks
           + (size_t)kStageBlocks * sizeof(unsigned short)           // tap / position of each staged block
           + (size_t)kStageBlocks * sizeof(unsigned)                 // round list
           + (kConvWaves + 1 + 2) * sizeof(int);
}

// Operands of one round = up to RB consecutive 16-pair blocks of ONE tap, fetched one round ahead of their use.
template <int KC, int NB, int RB>
struct RoundRegs {
    f32x4 a[RB][KC][2];     // A operand: lane holds x[in(pair 16j + jj)][kc*32 + 8*gq .. + 8)
    f32x4 b[KC][NB][2];     // B operand: lane holds w[tap][kc*32 + 8*gq + s][16*cb + jj], s = 0..7
    unsigned oaddr[RB][4];  // LDS byte address of accumulator (row of result row 4*gq + v, channel jj)
};

// Work split: each wave of the workgroup takes a contiguous share of the rounds.  A wave multiplies its blocks against the whole
// filter tap (all C_out channels), so an input row is fetched once per pair and a tap's weights once per round;
// the price is that two waves may add to the same accumulator, which the LDS fp64 atomic makes safe but not
// ordered: the fp64 sum can differ in its last bits from run to run.
// HALF: C_in = 16 (KC = 1): a lane's K slot gq stands for the four channels 4 gq .. 4 gq + 3 instead of eight, so a
// block takes four matrix instructions per 16 output channels and the second halves of the operands stay unused
// (the filter is prepared in the same 8-floats-per-lane layout, upper four zero).
template <int KC /* C_in / 32 */, int NB /* C_out / 16 */, int HALF = 0>
__global__ __launch_bounds__(kConvWaves * 64) void k_conv_mfma(int taps, long long nnz_in,
                                                               const float* __restrict__ feats,
                                                               const float* __restrict__ wb,
                                                               const float* __restrict__ bias,
                                                               const unsigned* __restrict__ pairs,
                                                               const unsigned short* __restrict__ block_tap,
                                                               const uint2* __restrict__ tile_hdr,
                                                               Counters* __restrict__ ctr,
                                                               float* __restrict__ resp) {
    static_assert(!HALF || KC == 1, "the half chunk stands alone");
    constexpr int C_IN = HALF ? 16 : KC * 32, C_OUT = NB * 16, CS = C_OUT + 1 /* padded accumulator row */;
    constexpr int RB = (KC * NB <= 4) ? 3 : ((KC * NB <= 8) ? 2 : 1);  // blocks per round
    constexpr int NT = kConvWaves * 64;
    static_assert(kStageBlocks % 4 == 0 && kStageBlocks <= 256, "stage size");
    extern __shared__ __align__(16) unsigned char smem[];
    double* s_c = (double*)smem;                                               // [129][CS]; row 128 absorbs padding
    unsigned* s_flat = (unsigned*)(s_c + (kTileRows + 1) * CS);                // [kStageBlocks][16] packed pairs
    unsigned short* s_btap = (unsigned short*)(s_flat + kStageBlocks * 16);    // [kStageBlocks]
    unsigned* s_rmeta = (unsigned*)(s_btap + kStageBlocks);  // [kStageBlocks] first block | blocks << 8 | tap << 16
    int* s_wlo = (int*)(s_rmeta + kStageBlocks);  // [kConvWaves + 1] first round of each wave; the last = all rounds
    int* s_next = s_wlo + kConvWaves + 1;         // [2] the workgroup's next tile (alternating slots)

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int jj = lane & 15, gq = lane >> 4;
    const unsigned long long lt_mask = (1ull << lane) - 1ull;
    const int n_tiles = (int)ctr->n_tiles;
    // LDS byte address of this lane's channel in accumulator row 0 (a generic pointer to LDS carries the LDS
    // address in its low 32 bits); accumulator addresses are formed once per block, at load time
    const unsigned lane_off = (unsigned)(size_t)s_c + (unsigned)jj * (unsigned)sizeof(double);

    // XCD-aware tile order: workgroup i runs on XCD i % kXcds; give each XCD one contiguous span of tiles so that
    // the input rows shared by neighbouring tiles stay in that XCD's L2.  Within its span a workgroup starts with
    // the tile of its slot and then draws tiles, in ascending order, from the span's counter (then from the other
    // spans' counters): tiles differ in work, and a fixed assignment would leave workgroups idle at the end.
    const int xcd = blockIdx.x % kXcds, slot = blockIdx.x / kXcds, per_xcd = gridDim.x / kXcds;
    const int span = (n_tiles + kXcds - 1) / kXcds;
    const int tile_end = (xcd + 1) * span < n_tiles ? (xcd + 1) * span : n_tiles;

    for (int i = threadIdx.x; i < kTileRows * CS; i += NT) s_c[i] = 0.0;  // the dummy row needs no reset
    // The stage buffer only ever holds entries written by the pair builder (or these zeros), so whatever a clamped
    // read past the end of a tile's list finds there names a valid input row.
    for (int i = threadIdx.x; i < kStageBlocks * 16; i += NT) s_flat[i] = 0u;

    int parity = 0;
    for (int tile = xcd * span + slot < tile_end ? xcd * span + slot : -1; tile >= 0; parity ^= 1) {
        const uint2 hdr = tile_hdr[tile];
        for (unsigned s0 = 0; s0 < hdr.y; s0 += kStageBlocks) {
            const int n_blocks = (int)((hdr.y - s0) < (unsigned)kStageBlocks ? (hdr.y - s0) : (unsigned)kStageBlocks);
            __syncthreads();  // previous stage consumed (and, for the first stage, the accumulators are zero)
            {   // ---- stage this tile's next blocks: a contiguous copy, 16 bytes per thread and step
                const uint4* src = (const uint4*)(pairs + (size_t)(hdr.x + s0) * 16);
                uint4* dst = (uint4*)s_flat;
                for (int i = threadIdx.x; i < n_blocks * 4; i += NT) dst[i] = src[i];
                for (int i = threadIdx.x; i < n_blocks; i += NT) s_btap[i] = block_tap[hdr.x + s0 + i];
            }
            __syncthreads();
            // ---- round list: a round = up to RB consecutive blocks of one tap.  It starts at every RB-th block of
            //      a tap's run (and at the start of the stage); entry = first block | blocks << 8 | tap << 16.
            //      Wave w takes the rounds that start in the w-th quarter of the stage's blocks: contiguous, and
            //      within one round of an even share of the blocks.
            if (wave == 0) {
                int base = 0;
                int lo[kConvWaves];
#pragma unroll
                for (int w = 0; w < kConvWaves; ++w) lo[w] = 0;
                for (int i0 = 0; i0 < n_blocks; i0 += 64) {
                    const int i = i0 + lane;
                    unsigned bt[RB];
#pragma unroll
                    for (int d = 0; d < RB; ++d) bt[d] = s_btap[(i + d) < n_blocks ? (i + d) : n_blocks - 1];
                    const bool start = i < n_blocks && (i == 0 || ((bt[0] >> 8) % RB) == 0);
                    int nb = 1;
#pragma unroll
                    for (int d = 1; d < RB; ++d)
                        if (nb == d && i + d < n_blocks && ((bt[d] >> 8) % RB) != 0) nb = d + 1;
                    const unsigned long long m = __ballot(start);
                    if (start)
                        s_rmeta[base + __popcll(m & lt_mask)] = (unsigned)i | (unsigned)nb << 8 | (bt[0] & 0xffu) << 16;
                    base += __popcll(m);
#pragma unroll
                    for (int w = 1; w < kConvWaves; ++w)  // rounds that start before the w-th share of the blocks
                        lo[w] += __popcll(__ballot(start && i * kConvWaves < w * n_blocks));
                }
                if (lane == 0) {
#pragma unroll
                    for (int w = 0; w < kConvWaves; ++w) s_wlo[w] = lo[w];
                    s_wlo[kConvWaves] = base;
                }
            }
            __syncthreads();
            const int r_lo = __builtin_amdgcn_readfirstlane(s_wlo[wave]);
            const int my_rounds = __builtin_amdgcn_readfirstlane(s_wlo[wave + 1]) - r_lo;
            if (my_rounds > 0) {
                // The wave's pipeline, per round: list entry (LDS) -> pair entries of its blocks (LDS) -> operands
                // (global) -> compute.  Each step is issued a full round before its result is needed, so that no
                // LDS or memory round trip sits between two rounds' matrix instructions.  All reads of a round are
                // unconditional, so that their number is fixed: a round past the end repeats the wave's last one
                // (never computed), a block past a round's end repeats list entries and is never computed.
                struct Entries {
                    unsigned in[RB];  // pair jj of each block (its input row)
                    uint4 out[RB];    // pairs 4*gq .. 4*gq + 3 of each block (their result rows)
                };
                auto meta_at = [&](int j) { return s_rmeta[r_lo + (j < my_rounds ? j : my_rounds - 1)]; };
                auto read_entries = [&](unsigned meta, Entries& E) {
                    const int first = (int)(meta & 0xffu);
#pragma unroll
                    for (int k = 0; k < RB; ++k) {
                        const int blk = (first + k) < kStageBlocks ? (first + k) : kStageBlocks - 1;
                        E.in[k] = s_flat[16 * blk + jj];
                        E.out[k] = *(const uint4*)(s_flat + 16 * blk + 4 * gq);
                    }
                };
                auto load_round = [&](unsigned meta, const Entries& E, RoundRegs<KC, NB, RB>& R) {
                    int tt = (int)((meta >> 16) & 0xffu);
                    tt = tt < taps ? tt : taps - 1;
                    const f32x4* wt = (const f32x4*)(wb + ((size_t)tt * KC * NB * 64 + lane) * 8);
#pragma unroll
                    for (int kc = 0; kc < KC; ++kc)
#pragma unroll
                        for (int cb = 0; cb < NB; ++cb) {
                            R.b[kc][cb][0] = wt[(kc * NB + cb) * 128];
                            if constexpr (!HALF) R.b[kc][cb][1] = wt[(kc * NB + cb) * 128 + 1];
                        }
#pragma unroll
                    for (int k = 0; k < RB; ++k) {
                        const unsigned in = E.in[k] & kPairInMask;
                        const f32x4* src = (const f32x4*)(feats + (size_t)in * C_IN + (HALF ? 4 : 8) * gq);
#pragma unroll
                        for (int kc = 0; kc < KC; ++kc) {
                            R.a[k][kc][0] = src[kc * 8];
                            if constexpr (!HALF) R.a[k][kc][1] = src[kc * 8 + 1];
                        }
                        // (a stale entry past the end of the list may name any row, but such a block is not computed)
                        R.oaddr[k][0] = (E.out[k].x >> kPairRowShift) * (unsigned)(CS * sizeof(double)) + lane_off;
                        R.oaddr[k][1] = (E.out[k].y >> kPairRowShift) * (unsigned)(CS * sizeof(double)) + lane_off;
                        R.oaddr[k][2] = (E.out[k].z >> kPairRowShift) * (unsigned)(CS * sizeof(double)) + lane_off;
                        R.oaddr[k][3] = (E.out[k].w >> kPairRowShift) * (unsigned)(CS * sizeof(double)) + lane_off;
                    }
                };
                // A block = NB independent fp32 MFMA chains per 32 input channels (one per 16 output channels); the
                // 16 x 16 results (rows = pairs 4*gq + v, column = channel 16*cb + jj) are added to the fp64
                // accumulators.  Padding pairs land in the dummy row.  Blocks are guarded one by one (uniform
                // branches) rather than through per-count variants, which the compiler would merge again through
                // scratch memory.
                auto compute_round = [&](unsigned meta, const RoundRegs<KC, NB, RB>& R) {
                    const int nb = (int)((meta >> 8) & 0xffu);  // 1 .. RB
#pragma unroll
                    for (int k = 0; k < RB; ++k) {
                        if (k == 0 || k < nb) {  // (a round has at least one block)
#pragma unroll
                            for (int kc = 0; kc < KC; ++kc) {
                                f32x4 acc[NB];
#pragma unroll
                                for (int cb = 0; cb < NB; ++cb) {
                                    f32x4 c = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                                    for (int s = 0; s < 4; ++s)
                                        c = __builtin_amdgcn_mfma_f32_16x16x4f32(R.a[k][kc][0][s], R.b[kc][cb][0][s], c, 0, 0, 0);
                                    if constexpr (!HALF) {
#pragma unroll
                                        for (int s = 0; s < 4; ++s)
                                            c = __builtin_amdgcn_mfma_f32_16x16x4f32(R.a[k][kc][1][s], R.b[kc][cb][1][s], c, 0, 0, 0);
                                    }
                                    acc[cb] = c;
                                }
#pragma unroll
                                for (int cb = 0; cb < NB; ++cb)
#pragma unroll
                                    for (int v = 0; v < 4; ++v)
                                        __hip_atomic_fetch_add(
                                            (__attribute__((address_space(3))) double*)(size_t)R.oaddr[k][v] + cb * 16,
                                            (double)acc[cb][v], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                            }
                        }
                    }
                };
                RoundRegs<KC, NB, RB> r0, r1;
                Entries ent;
                unsigned m0 = __builtin_amdgcn_readfirstlane(meta_at(0));
                unsigned m1 = __builtin_amdgcn_readfirstlane(meta_at(1));
                unsigned m_ahead = meta_at(2);
                read_entries(m0, ent);
                load_round(m0, ent, r0);
                read_entries(m1, ent);
                // Let these first reads land before the loop: inside it, every value read from LDS is used only
                // after a round's worth of accumulator updates has been issued behind the read, so the wait for
                // it (the LDS queue is in order) does not wait for those updates.
                asm volatile("" : "+v"(m_ahead));
#pragma unroll
                for (int k = 0; k < RB; ++k)
                    asm volatile("" : "+v"(ent.in[k]), "+v"(ent.out[k].x), "+v"(ent.out[k].y), "+v"(ent.out[k].z),
                                 "+v"(ent.out[k].w));
                for (int j = 0; j < my_rounds; j += 2) {
                    // here: r0 = operands of round j (list entry m0), ent = pair entries of round j + 1 (m1),
                    //       m_ahead = list entry of round j + 2
                    load_round(m1, ent, r1);
                    const unsigned m2 = __builtin_amdgcn_readfirstlane(m_ahead);
                    read_entries(m2, ent);
                    m_ahead = meta_at(j + 3);
                    compute_round(m0, r0);
                    if (j + 1 >= my_rounds) break;
                    load_round(m2, ent, r0);
                    const unsigned m3 = __builtin_amdgcn_readfirstlane(m_ahead);
                    read_entries(m3, ent);
                    m_ahead = meta_at(j + 4);
                    compute_round(m1, r1);
                    m0 = m2;
                    m1 = m3;
                }
            }
        }
        // Draw the next tile: from the own span, and once that is used up from the other spans, so that no XCD ends
        // before the others.  The last wave does it when its share of the tile is done: it has the smallest share
        // on average and would otherwise only wait at the barrier, which hides the atomic's round trip.
        if (threadIdx.x == NT - 64) {
            int t = -1;
            for (int d = 0; d < kXcds && t < 0; ++d) {
                const int x = (xcd + d) % kXcds;
                const int end_x = (x + 1) * span < n_tiles ? (x + 1) * span : n_tiles;
                if (x * span + per_xcd >= end_x) continue;  // (a span with no tiles to draw)
                const int cand = x * span + per_xcd + (int)atomicAdd(&ctr->conv_ticket[x * kTicketStride], 1u);
                if (cand < end_x) t = cand;
            }
            s_next[parity] = t;
        }
        __syncthreads();
        const int next_tile = s_next[parity];
        // ---- epilogue: one rounding to fp32, bias on the non-zero entries, planar store; the accumulators are
        //      reset on the way.  A lane takes one row, a wave one channel at a time: consecutive rows lie
        //      CS doubles apart, i.e. 2 banks (mod 64), so the 64 reads of a wave spread over all LDS banks, and
        //      the wave's stores form one contiguous 256-byte run of the planar tile.
        {
            constexpr int OCW = (C_OUT + kConvWaves - 1) / kConvWaves, H = kTileRows / 64;
            double acc[OCW][H];
#pragma unroll
            for (int j = 0; j < OCW; ++j) {  // all reads first: one LDS latency for the lot
                const int oc = (wave + j * kConvWaves) < C_OUT ? (wave + j * kConvWaves) : C_OUT - 1;
#pragma unroll
                for (int h = 0; h < H; ++h) acc[j][h] = s_c[(h * 64 + lane) * CS + oc];
            }
#pragma unroll
            for (int j = 0; j < OCW; ++j) {
                const int oc = wave + j * kConvWaves;
                if (C_OUT % kConvWaves == 0 || oc < C_OUT) {
                    // (the weights stand in as a readable address when there is no bias)
                    const float bl = (bias ? bias : wb)[oc];
                    const float bv = bias ? bl : 0.0f;
#pragma unroll
                    for (int h = 0; h < H; ++h) {
                        const int r = h * 64 + lane;
                        s_c[r * CS + oc] = 0.0;
                        float x = (float)acc[j][h];
                        if (x != 0.0f) x += bv;
                        resp[((size_t)tile * C_OUT + oc) * kTileRows + r] = x;
                    }
                }
            }
        }
        tile = next_tile;
    }
}

template <int KC, int NB, int HALF = 0>
static hipError_t launch_conv_mfma_t(int taps, long long nnz_in, const float* feats, const float* wb, const float* bias,
                                     const unsigned* pairs, const unsigned short* block_tap, const uint2* tile_hdr,
                                     Counters* ctr, float* resp, hipStream_t s) {
    const size_t lds = conv_mfma_lds_bytes(NB * 16);
    // (set on every launch: the attribute belongs to the current device's copy of the kernel, and a flag remembering
    // that it was set would have to be kept per device and guarded between threads for the sake of a microsecond)
    hipError_t e = hipFuncSetAttribute((const void*)k_conv_mfma<KC, NB, HALF>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    int per_cu = (int)((160 * 1024) / lds);
    if (per_cu < 1) per_cu = 1;
    if (per_cu > 4) per_cu = 4;    // 16 waves per CU
    const int grid = (device_cu_count() * per_cu + kXcds - 1) / kXcds * kXcds;  // one span of tiles per XCD
    hipLaunchKernelGGL((k_conv_mfma<KC, NB, HALF>), dim3(grid), dim3(kConvWaves * 64), lds, s, taps, nnz_in, feats, wb,
                       bias,
                       pairs, block_tap, tile_hdr, ctr, resp);
    return hipGetLastError();
}

bool conv_mfma_supported(const Geom& g, int c_in, int c_out, long long nnz_in) {
    if (g.T > 255) return false;  // block_tap holds the tap in one byte
    return ((c_in % 32 == 0 && c_in <= 128) || c_in == 16) && c_out % 16 == 0 && c_out <= 64 && nnz_in > 0 &&
           nnz_in < (1ll << kPairRowShift);
}

hipError_t launch_conv_mfma(const Geom& g, long long nnz_in, const float* feats, int c_in, const float* wb, int c_out,
                            const float* bias, const unsigned* pairs, const unsigned short* block_tap,
                            const uint2* tile_hdr, Counters* ctr, float* resp, hipStream_t s) {
#define SCNN_MFMA_CASE(KC_, NB_)                                                                                  \
    if (c_in == KC_ * 32 && c_out == NB_ * 16)                                                                    \
        return launch_conv_mfma_t<KC_, NB_>(g.T, nnz_in, feats, wb, bias, pairs, block_tap, tile_hdr, ctr, resp, s);
    SCNN_MFMA_CASE(1, 1) SCNN_MFMA_CASE(1, 2) SCNN_MFMA_CASE(1, 3) SCNN_MFMA_CASE(1, 4)
    SCNN_MFMA_CASE(2, 1) SCNN_MFMA_CASE(2, 2) SCNN_MFMA_CASE(2, 3) SCNN_MFMA_CASE(2, 4)
    SCNN_MFMA_CASE(3, 1) SCNN_MFMA_CASE(3, 2) SCNN_MFMA_CASE(3, 3) SCNN_MFMA_CASE(3, 4)
    SCNN_MFMA_CASE(4, 1) SCNN_MFMA_CASE(4, 2) SCNN_MFMA_CASE(4, 3) SCNN_MFMA_CASE(4, 4)
#undef SCNN_MFMA_CASE
#define SCNN_MFMA_HALF(NB_)                                                                                       \
    if (c_in == 16 && c_out == NB_ * 16)                                                                          \
        return launch_conv_mfma_t<1, NB_, 1>(g.T, nnz_in, feats, wb, bias, pairs, block_tap, tile_hdr, ctr, resp, s);
    SCNN_MFMA_HALF(1) SCNN_MFMA_HALF(2) SCNN_MFMA_HALF(3) SCNN_MFMA_HALF(4)
#undef SCNN_MFMA_HALF
    return hipErrorInvalidValue;
}

}  // namespace scnn
