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
#include "scnn_internal.h"

namespace scnn {

constexpr int kTapChunk = 32;  // taps whose neighbour rows are staged in LDS at a time
constexpr int kOcBlock = 16;   // output channels accumulated per thread

// Generic vector kernel: any C_in, C_out, any filter sparsity.
// Work item = (tile, block of 32 output channels); thread = (row, 16 channels).
__global__ __launch_bounds__(256) void k_conv_valu(Geom g, const unsigned long long* __restrict__ occ,
                                                   const unsigned* __restrict__ occ_prefix, long long nnz_in,
                                                   const float* __restrict__ feats, int c_in,
                                                   const double* __restrict__ wp, int c_out, int c_out_pad,
                                                   const float* __restrict__ bias,
                                                   const int* __restrict__ tap_active,
                                                   const unsigned* __restrict__ cand_lin,
                                                   const int* __restrict__ cand_start,
                                                   const int* __restrict__ tile_start,
                                                   const Counters* __restrict__ ctr, float* __restrict__ resp) {
    __shared__ int s_nbr[kTileRows][kTapChunk + 1];
    __shared__ int s_site[kTileRows][3];

    const int n_tiles = (int)ctr->n_tiles;
    const int n_chunks = (c_out_pad + 2 * kOcBlock - 1) / (2 * kOcBlock);
    const long long n_items = (long long)n_tiles * n_chunks;
    const int row = threadIdx.x & (kTileRows - 1);
    const int half = __builtin_amdgcn_readfirstlane(threadIdx.x >> 7);  // which 16-channel block of the chunk

    for (long long item = blockIdx.x; item < n_items; item += gridDim.x) {
        const int tile = (int)(item / n_chunks);
        const int chunk = (int)(item - (long long)tile * n_chunks);
        const int b = sample_of_tile(tile_start, g.batch, tile);
        const int first = cand_start[b] + (tile - tile_start[b]) * kTileRows;
        int nrows = cand_start[b + 1] - first;
        if (nrows > kTileRows) nrows = kTileRows;
        const int oc0 = chunk * 2 * kOcBlock + half * kOcBlock;
        const bool oc_valid = oc0 < c_out_pad;

        __syncthreads();  // previous item's readers of s_site / s_nbr are done
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

        for (int tc = 0; tc < g.T; tc += kTapChunk) {
            __syncthreads();
            for (int i = threadIdx.x; i < kTileRows * kTapChunk; i += 256) {
                const int tt = i & (kTapChunk - 1), r = i >> 5;
                const int t = tc + tt;
                int n = -1;
                if (t < g.T && r < nrows && tap_active[t]) {
                    const int t2 = t % g.K[2], t1 = (t / g.K[2]) % g.K[1], t0 = t / (g.K[2] * g.K[1]);
                    n = lookup_row(g, occ, occ_prefix, nnz_in, b, s_site[r][0] + t0 - g.H[0],
                                   s_site[r][1] + t1 - g.H[1], s_site[r][2] + t2 - g.H[2]);
                }
                s_nbr[r][tt] = n;
            }
            __syncthreads();
            if (oc_valid && row < nrows) {
                const int tmax = (g.T - tc) < kTapChunk ? (g.T - tc) : kTapChunk;
                for (int tt = 0; tt < tmax; ++tt) {
                    const int n = s_nbr[row][tt];
                    if (n < 0) continue;
                    const float* __restrict__ x = feats + (size_t)n * c_in;
                    const double* __restrict__ wt = wp + ((size_t)(tc + tt) * c_in) * c_out_pad + oc0;
                    for (int ic = 0; ic < c_in; ++ic) {
                        const double xv = (double)x[ic];
                        const double* __restrict__ wr = wt + (size_t)ic * c_out_pad;
#pragma unroll
                        for (int o = 0; o < kOcBlock; ++o) acc[o] = fma(xv, wr[o], acc[o]);
                    }
                }
            }
        }
        if (oc_valid) {
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

hipError_t launch_conv_valu(const Geom& g, const unsigned long long* occ, const unsigned* occ_prefix,
                            long long nnz_in, const float* feats, int c_in, const double* wp, int c_out,
                            int c_out_pad, const float* bias, const int* tap_active, const unsigned* cand_lin,
                            const int* cand_start, const int* tile_start, const Counters* ctr, float* resp,
                            hipStream_t s) {
    hipLaunchKernelGGL(k_conv_valu, dim3(256 * 8), dim3(256), 0, s, g, occ, occ_prefix, nnz_in, feats, c_in, wp,
                       c_out, c_out_pad, bias, tap_active, cand_lin, cand_start, tile_start, ctr, resp);
    return hipGetLastError();
}

}  // namespace scnn
