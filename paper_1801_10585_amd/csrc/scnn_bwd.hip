// Back-propagation through the convolution (Algorithm 2, with the masks of Eq. 3).
//
// The paper walks the same loop nest as the forward pass and issues two atomic
// adds per multiply (one into bp_data, one into bp_filter).  Here both outputs
// are formed without value atomics:
//
//   bp_data[q, ic]      = sum over taps t, channels oc of  w[t, ic, oc] * g[q - delta_t, oc]     (x[q, ic] != 0)
//   bp_filter[t, ic, oc] = sum over input rows q of         x[q, ic]    * g[q - delta_t, oc]     (w[t, ic, oc] != 0)
//
// bp_data is the forward convolution of the gradient rows with the adjoint
// filter (taps negated, channels transposed), evaluated at the input's own
// sites only: the forward kernels are reused with the input rows as the list
// of output sites (gather form, fixed summation order in the vector kernel).
// bp_filter is a reduction over (input row, gradient row) pairs per tap: every
// workgroup (vector kernel) or wave (matrix-core kernel) sums a share of the
// tiles into a private partial filter in fp64 and stores it; a last kernel
// adds the partials in a fixed order, applies the mask and rounds to fp32 once.
#include "scnn_internal.h"

namespace scnn {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kBwdTapChunk = 32;  // taps whose neighbour rows are staged in LDS at a time (vector kernel)

// ------------------------------------------------------------------ input rows as the list of output sites
// cand_lin[r] = site index of input row r; rows16_start[b] = 16-row groups of all earlier samples (the unit in
// which the pair lists reserve their space).  Rows outside the grid or out of order are reported.
__global__ __launch_bounds__(256) void k_bwd_sites(Geom g, const int32_t* __restrict__ coords, long long rows,
                                                   const int* __restrict__ cand_start,
                                                   unsigned* __restrict__ cand_lin, int* __restrict__ rows16_start,
                                                   Counters* ctr) {
    const int stride = 1 + g.ndim;
    for (long long r = (long long)blockIdx.x * blockDim.x + threadIdx.x; r < rows;
         r += (long long)gridDim.x * blockDim.x) {
        int b, c0, c1, c2;
        load_site(g, coords + r * stride, b, c0, c1, c2);
        unsigned lin = 0;
        if (site_in_grid(g, b, c0, c1, c2)) {
            lin = (unsigned)lin_of(g, c0, c1, c2);
            if (r > 0) {
                int pb, p0, p1, p2;
                load_site(g, coords + (r - 1) * stride, pb, p0, p1, p2);
                if (site_in_grid(g, pb, p0, p1, p2) &&
                    (long long)pb * g.Npad + lin_of(g, p0, p1, p2) >= (long long)b * g.Npad + lin)
                    atomicOr(&ctr->flags, SCNN_FLAG_UNSORTED);
            }
        } else {
            atomicOr(&ctr->flags, SCNN_FLAG_BAD_COORD);
        }
        cand_lin[r] = lin;
    }
    if (blockIdx.x == 0) {  // (whole block)
        __shared__ unsigned s_wave[4];
        (void)sample_ranges_256(g.batch, cand_start, nullptr, rows16_start, s_wave);
    }
}

hipError_t launch_bwd_sites(const Geom& g, const int32_t* coords, long long rows, const int* cand_start,
                            unsigned* cand_lin, int* rows16_start, Counters* ctr, hipStream_t s) {
    long long blocks = (rows + 255) / 256;
    if (blocks < 1) blocks = 1;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(k_bwd_sites, dim3((unsigned)blocks), dim3(256), 0, s, g, coords, rows, cand_start, cand_lin,
                       rows16_start, ctr);
    return hipGetLastError();
}

// ------------------------------------------------------------------ bp_data: planar tiles -> rows, masked by x != 0
// resp[tile][ic][row] holds the adjoint convolution at the input rows of the tile (Eq. 3, first line: the
// gradient reaches non-zero input values only).  Through LDS so that both sides coalesce.
__global__ __launch_bounds__(256) void k_bwd_data_write(Geom g, const float* __restrict__ resp,
                                                        const float* __restrict__ x, int c_in,
                                                        const int* __restrict__ cand_start,
                                                        const int* __restrict__ tile_start,
                                                        const Counters* __restrict__ ctr,
                                                        float* __restrict__ bp_data) {
    __shared__ float s_t[kTileRows][65];
    const int n_tiles = (int)ctr->n_tiles;
    // rows of x and bp_data start on 16-byte boundaries
    const bool vec4 = (c_in & 3) == 0 && ((((size_t)x) | ((size_t)bp_data)) & 15) == 0;
    for (int tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const int b = sample_of_tile(tile_start, g.batch, tile);
        const int first = cand_start[b] + (tile - tile_start[b]) * kTileRows;
        int nrows = cand_start[b + 1] - first;
        if (nrows > kTileRows) nrows = kTileRows;
        for (int cc = 0; cc < c_in; cc += 64) {
            const int cw = (c_in - cc) < 64 ? (c_in - cc) : 64;
            __syncthreads();
            for (int i = threadIdx.x; i < kTileRows * cw; i += 256) {
                const int c = i >> 7, r = i & 127;
                s_t[r][c] = resp[((size_t)tile * c_in + cc + c) * kTileRows + r];
            }
            __syncthreads();
            if (vec4) {  // four channels per thread: 16-byte loads of x and stores of bp_data
                const int q = cw >> 2;
                for (int i = threadIdx.x; i < nrows * q; i += 256) {
                    const int r = i / q, c = (i - r * q) * 4;
                    const size_t at = (size_t)(first + r) * c_in + cc + c;
                    const float4 xv = *reinterpret_cast<const float4*>(x + at);
                    float4 o;
                    o.x = xv.x != 0.0f ? s_t[r][c] : 0.0f;
                    o.y = xv.y != 0.0f ? s_t[r][c + 1] : 0.0f;
                    o.z = xv.z != 0.0f ? s_t[r][c + 2] : 0.0f;
                    o.w = xv.w != 0.0f ? s_t[r][c + 3] : 0.0f;
                    *reinterpret_cast<float4*>(bp_data + at) = o;
                }
            } else {
                for (int i = threadIdx.x; i < nrows * cw; i += 256) {
                    const int r = i / cw, c = i - r * cw;
                    const size_t at = (size_t)(first + r) * c_in + cc + c;
                    bp_data[at] = (x[at] != 0.0f) ? s_t[r][c] : 0.0f;
                }
            }
        }
    }
}

hipError_t launch_bwd_data_write(const Geom& g, const float* resp, const float* x, int c_in, const int* cand_start,
                                 const int* tile_start, const Counters* ctr, long long tiles_cap, float* bp_data,
                                 hipStream_t s) {
    long long blocks = tiles_cap < 1 ? 1 : (tiles_cap > 4096 ? 4096 : tiles_cap);
    hipLaunchKernelGGL(k_bwd_data_write, dim3((unsigned)blocks), dim3(256), 0, s, g, resp, x, c_in, cand_start,
                       tile_start, ctr, bp_data);
    return hipGetLastError();
}

// ------------------------------------------------------------------ bp_filter, vector kernel (any shape)
// Work item = (block of 256 consecutive filter elements in [t][ic][oc] order, share of the tiles).  A thread owns
// one element and walks the rows of its tiles: row q contributes x[q, ic] * g[q - delta_t, oc] when the gradient
// has a row at q - delta_t.  The neighbour rows of a tile are looked up once per tap and shared through LDS.
// fp64 throughout; the partial sum of the share is stored (no atomics), zero included.
__global__ __launch_bounds__(256) void k_bwd_filter_valu(Geom g, const unsigned long long* __restrict__ occ,
                                                         const unsigned* __restrict__ occ_prefix, long long g_rows,
                                                         const float* __restrict__ gf, int c_out,
                                                         const float* __restrict__ x, int c_in,
                                                         const int* __restrict__ tap_active /* adjoint tap order */,
                                                         const unsigned* __restrict__ cand_lin,
                                                         const int* __restrict__ cand_start,
                                                         const int* __restrict__ tile_start,
                                                         const Counters* __restrict__ ctr, int n_eb, int n_chunks,
                                                         double* __restrict__ fpart) {
    __shared__ int s_nbr[kTileRows][kBwdTapChunk + 1];
    __shared__ int s_site[kTileRows][3];
    const int n_tiles = (int)ctr->n_tiles;
    const int cc = c_in * c_out;
    const long long n_elem = (long long)g.T * cc;
    const int eb = (int)(blockIdx.x % (unsigned)n_eb), chunk = (int)(blockIdx.x / (unsigned)n_eb);
    const long long e = (long long)eb * 256 + threadIdx.x;
    const bool valid = e < n_elem;
    const int t_e = valid ? (int)(e / cc) : -1;
    const int ic = valid ? (int)((e % cc) / c_out) : 0, oc = valid ? (int)(e % c_out) : 0;
    const int t_lo = (int)(((long long)eb * 256) / cc);
    long long e_hi = (long long)eb * 256 + 255;
    if (e_hi > n_elem - 1) e_hi = n_elem - 1;
    const int t_hi = (int)(e_hi / cc);
    double acc = 0.0;

    for (int tile = chunk; tile < n_tiles; tile += n_chunks) {
        const int b = sample_of_tile(tile_start, g.batch, tile);
        const int first = cand_start[b] + (tile - tile_start[b]) * kTileRows;
        int nrows = cand_start[b + 1] - first;
        if (nrows > kTileRows) nrows = kTileRows;
        __syncthreads();  // readers of s_site / s_nbr of the previous tile are done
        if (threadIdx.x < kTileRows) {
            int c0 = 0, c1 = 0, c2 = 0;
            if (threadIdx.x < nrows) site_of(g, cand_lin[first + threadIdx.x], c0, c1, c2);
            s_site[threadIdx.x][0] = c0;
            s_site[threadIdx.x][1] = c1;
            s_site[threadIdx.x][2] = c2;
        }
        for (int tc = t_lo; tc <= t_hi; tc += kBwdTapChunk) {
            __syncthreads();
            // The gradient row of (row, tap t) sits at site - delta_t = site + delta of the mirrored tap T-1-t, so the
            // look-ups run over the mirrored (adjoint) tap indices, per filter line: the taps of a line look at
            // adjacent sites and share one pair of bitmap words.  tap_active is in adjoint order already.
            {
                const int t_last = (tc + kBwdTapChunk - 1) < t_hi ? (tc + kBwdTapChunk - 1) : t_hi;
                const int a_lo = g.T - 1 - t_last, a_hi = g.T - 1 - tc;  // adjoint taps [a_lo, a_hi]
                const int l_first = a_lo / g.K[2];
                const int n_seg = a_hi / g.K[2] - l_first + 1;
                for (int i = threadIdx.x; i < kTileRows * n_seg; i += 256) {
                    const int r = i & (kTileRows - 1), l = l_first + (i >> 7);
                    const int aa = a_lo > l * g.K[2] ? a_lo : l * g.K[2];
                    const int ab = (a_hi + 1) < (l + 1) * g.K[2] ? (a_hi + 1) : (l + 1) * g.K[2];
                    const int t0 = l / g.K[1], t1 = l - t0 * g.K[1];
                    int* dst = &s_nbr[r][0];
                    lookup_line(g, occ, occ_prefix, g_rows, r < nrows, b, s_site[r][0], s_site[r][1], s_site[r][2], t0,
                                t1, aa - l * g.K[2], ab - aa, tap_active + aa,
                                [&](int k, int n) { dst[g.T - 1 - (aa + k) - tc] = n; });
                }
            }
            __syncthreads();
            if (valid && t_e >= tc && t_e < tc + kBwdTapChunk) {
                const int tt = t_e - tc;
                // eight rows at a time, their loads independent of one another; the sum keeps the row order
                for (int r0 = 0; r0 < nrows; r0 += 8) {
                    float xv[8], gv[8];
                    bool on[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const int r = r0 + u;
                        const int n = r < nrows ? s_nbr[r][tt] : -1;
                        on[u] = n >= 0;
                        xv[u] = x[(size_t)(first + (r < nrows ? r : 0)) * c_in + ic];
                        gv[u] = on[u] ? gf[(size_t)n * c_out + oc] : 0.0f;  // (no gradient row: nothing is read)
                    }
#pragma unroll
                    for (int u = 0; u < 8; ++u)
                        if (on[u]) acc = fma((double)xv[u], (double)gv[u], acc);
                }
            }
        }
    }
    if (valid) fpart[(size_t)chunk * n_elem + e] = acc;
}

hipError_t launch_bwd_filter_valu(const Geom& g, const unsigned long long* occ, const unsigned* occ_prefix,
                                  long long g_rows, const float* gf, int c_out, const float* x, int c_in,
                                  const int* tap_active, const unsigned* cand_lin, const int* cand_start,
                                  const int* tile_start, const Counters* ctr, int n_chunks, double* fpart,
                                  hipStream_t s) {
    const long long n_elem = (long long)g.T * c_in * c_out;
    const int n_eb = (int)((n_elem + 255) / 256);
    hipLaunchKernelGGL(k_bwd_filter_valu, dim3((unsigned)((long long)n_eb * n_chunks)), dim3(256), 0, s, g, occ,
                       occ_prefix, g_rows, gf, c_out, x, c_in, tap_active, cand_lin, cand_start, tile_start, ctr,
                       n_eb, n_chunks, fpart);
    return hipGetLastError();
}

// ------------------------------------------------------------------ bp_filter, matrix-core kernel
// Uses the pair lists of the adjoint convolution: per tile of 128 input rows and per adjoint tap t', blocks of 16
// (local input row, gradient row) pairs.  For one tap the filter gradient is the contraction
//     D[ic][oc] += sum over pairs  x[q(pair)][ic] * g[p(pair)][oc],
// i.e. a [C_in x pairs] . [pairs x C_out] product whose long dimension is the pair list: the pairs are the K
// dimension of v_mfma_f32_16x16x4_f32, four per instruction.  A wave owns one (tap, 16*MT input channels,
// 16*NT output channels) slab and a contiguous share of the tiles; it keeps the slab in registers for its whole
// life: fp32 matrix-core sums over the (at most 128) pairs of one tile, added to an fp64 copy after each tile.
// Lane (jj = lane & 15, gq = lane >> 4) feeds pair 4*gq + j of a block in step j (the order of the pairs inside a
// sum is free), input channels jj*MT + i and output channels jj*NT + i of the slab, so that its operands are one
// 8- or 16-byte load per pair at a 32-bit offset from a wave-uniform base: three vector instructions of address
// arithmetic per pair.  Only the last block of a tap can hold list padding (local row 128), so only that block
// pays for masking.
//
// All slabs of one share of the tiles run on the same XCD (workgroup i runs on XCD i % 8), so that the share's
// input rows and gradient rows are fetched into that XCD's L2 once for all taps.
template <int MT, int NT>
struct BwdOperands {
    float av[4][MT], bv[4][NT];
};

template <int MT, int NT, bool MASKED>
__device__ __forceinline__ void bwd_filter_load(const uint4 ent, const char* __restrict__ xt,
                                                const char* __restrict__ gl, unsigned cin4, unsigned cout4,
                                                unsigned xlane, unsigned glane, BwdOperands<MT, NT>& o) {
    const unsigned en[4] = {ent.x, ent.y, ent.z, ent.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const unsigned row = en[j] >> kPairRowShift;
        // the 24-bit multiply reads the low 24 bits of its operands: the gradient row of the pair, as it is
        const unsigned goff = __umul24(en[j], cout4) + glane;
        unsigned xoff = __umul24(row, cin4) + xlane;
        bool live = true;
        if constexpr (MASKED) {
            live = row < (unsigned)kTileRows;
            xoff = live ? xoff : xlane;
        }
        if constexpr (MT == 1) {
            o.av[j][0] = *(const float*)(xt + xoff);
        } else {
            const float2 t2 = *(const float2*)(xt + xoff);
            o.av[j][0] = t2.x;
            o.av[j][1] = t2.y;
        }
        if constexpr (MASKED) {
#pragma unroll
            for (int a = 0; a < MT; ++a) o.av[j][a] = live ? o.av[j][a] : 0.0f;
        }
        if constexpr (NT == 1) {
            o.bv[j][0] = *(const float*)(gl + goff);
        } else if constexpr (NT == 2) {
            const float2 t2 = *(const float2*)(gl + goff);
            o.bv[j][0] = t2.x;
            o.bv[j][1] = t2.y;
        } else {
            const float4 t4 = *(const float4*)(gl + goff);
            o.bv[j][0] = t4.x;
            o.bv[j][1] = t4.y;
            o.bv[j][2] = t4.z;
            o.bv[j][3] = t4.w;
        }
    }
}

template <int MT, int NT>
__device__ __forceinline__ void bwd_filter_mma(const BwdOperands<MT, NT>& o, f32x4 (&acc)[MT][NT]) {
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int a = 0; a < MT; ++a)
#pragma unroll
            for (int c = 0; c < NT; ++c)
                acc[a][c] = __builtin_amdgcn_mfma_f32_16x16x4f32(o.av[j][a], o.bv[j][c], acc[a][c], 0, 0, 0);
}

template <int MT, int NT>
__global__ __launch_bounds__(256) void k_bwd_filter_mfma(int taps, int c_in, int c_out, const float* __restrict__ x,
                                                         const float* __restrict__ gf,
                                                         const unsigned* __restrict__ pairs,
                                                         const unsigned short* __restrict__ tap_first,
                                                         const uint2* __restrict__ tile_hdr,
                                                         const int* __restrict__ cand_start,
                                                         const int* __restrict__ tile_start, int batch,
                                                         const Counters* __restrict__ ctr, int n_chunks,
                                                         int groups /* workgroups per share */,
                                                         double* __restrict__ fpart) {
    const int lane = threadIdx.x & 63;
    const int jj = lane & 15, gq = lane >> 4;
    const int n_icb = c_in / (16 * MT), n_ocb = c_out / (16 * NT);
    const int slabs = taps * n_icb * n_ocb;
    const int xcd = blockIdx.x % kXcds, j_in_xcd = blockIdx.x / kXcds;
    const int chunk = (j_in_xcd / groups) * kXcds + xcd;
    const int slab = __builtin_amdgcn_readfirstlane((j_in_xcd % groups) * 4 + (int)(threadIdx.x >> 6));
    if (chunk >= n_chunks || slab >= slabs) return;
    const int ta = slab / (n_icb * n_ocb);  // adjoint tap
    const int icb = (slab / n_ocb) % n_icb, ocb = slab % n_ocb;
    const int n_tiles = (int)ctr->n_tiles;
    // contiguous share of the tiles
    const int tile_lo = (int)((long long)chunk * n_tiles / n_chunks);
    const int tile_hi = (int)((long long)(chunk + 1) * n_tiles / n_chunks);
    const unsigned cin4 = (unsigned)c_in * 4u, cout4 = (unsigned)c_out * 4u;
    const unsigned xlane = (unsigned)(icb * 16 * MT + jj * MT) * 4u, glane = (unsigned)(ocb * 16 * NT + jj * NT) * 4u;
    const char* __restrict__ gl = (const char*)gf;

    double acc64[MT][NT][4];
#pragma unroll
    for (int a = 0; a < MT; ++a)
#pragma unroll
        for (int c = 0; c < NT; ++c)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc64[a][c][v] = 0.0;

    int b = tile_lo < tile_hi ? sample_of_tile(tile_start, batch, tile_lo) : 0;
    int b_end = tile_start[b + 1];  // first tile of the next sample
    // block range of this tap in a tile; fetched one tile ahead of its use
    unsigned nb0 = 0, nb1 = 0;
    if (tile_lo < tile_hi) {
        const unsigned short* tf = tap_first + (size_t)tile_lo * (taps + 1) + ta;
        const unsigned h = tile_hdr[tile_lo].x;
        nb0 = h + tf[0];
        nb1 = h + tf[1];
    }
    for (int tile = tile_lo; tile < tile_hi; ++tile) {
        const unsigned b0 = nb0, b1 = nb1;
        if (tile + 1 < tile_hi) {
            const unsigned short* tf = tap_first + (size_t)(tile + 1) * (taps + 1) + ta;
            const unsigned h = tile_hdr[tile + 1].x;
            nb0 = h + tf[0];
            nb1 = h + tf[1];
        }
        while (tile >= b_end) {  // next sample (samples without rows have no tiles)
            ++b;
            b_end = tile_start[b + 1];
        }
        if (b0 >= b1) continue;
        const int first = cand_start[b] + (tile - tile_start[b]) * kTileRows;
        const char* __restrict__ xt = (const char*)(x + (size_t)first * c_in);
        f32x4 acc[MT][NT];
#pragma unroll
        for (int a = 0; a < MT; ++a)
#pragma unroll
            for (int c = 0; c < NT; ++c) acc[a][c] = f32x4{0.f, 0.f, 0.f, 0.f};
        // operands one block ahead of their use (two register sets that swap roles, so that nothing is copied),
        // pair entries two blocks ahead
        const unsigned* pl = pairs + (size_t)b0 * 16 + gq * 4;
        const unsigned nblk = b1 - b0;
        BwdOperands<MT, NT> opa, opb;
        uint4 ent_next = *(const uint4*)pl;
        unsigned issued = 0, done = 0;
        auto issue = [&](BwdOperands<MT, NT>& dst) {
            const uint4 e = ent_next;
            if (issued + 1 < nblk) ent_next = *(const uint4*)(pl + (size_t)(issued + 1) * 16);
            if (issued + 1 < nblk)
                bwd_filter_load<MT, NT, false>(e, xt, gl, cin4, cout4, xlane, glane, dst);
            else
                bwd_filter_load<MT, NT, true>(e, xt, gl, cin4, cout4, xlane, glane, dst);
            ++issued;
        };
        issue(opa);
        for (;;) {
            if (issued < nblk) issue(opb);
            bwd_filter_mma<MT, NT>(opa, acc);
            if (++done == nblk) break;
            if (issued < nblk) issue(opa);
            bwd_filter_mma<MT, NT>(opb, acc);
            if (++done == nblk) break;
        }
#pragma unroll
        for (int a = 0; a < MT; ++a)
#pragma unroll
            for (int c = 0; c < NT; ++c)
#pragma unroll
                for (int v = 0; v < 4; ++v) acc64[a][c][v] = fma((double)acc[a][c][v], 1.0, acc64[a][c][v]);  // full-rate form of the add
    }
    // result element (a, c, v) of this lane: input channel (4*gq + v)*MT + a, output channel jj*NT + c of the slab
    const int t = taps - 1 - ta;  // tap of the filter itself
    double* out = fpart + ((size_t)chunk * taps + t) * c_in * c_out;
#pragma unroll
    for (int a = 0; a < MT; ++a)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int ic = icb * 16 * MT + (4 * gq + v) * MT + a;
#pragma unroll
            for (int c = 0; c < NT; ++c) out[(size_t)ic * c_out + ocb * 16 * NT + jj * NT + c] = acc64[a][c][v];
        }
}

// The gradient values are addressed with 32-bit byte offsets.
bool bwd_filter_mfma_supported(int c_in, int c_out, long long g_rows) {
    return c_in % 16 == 0 && c_out % 16 == 0 && g_rows * c_out * 4 < (1ll << 32);
}

// waves per share of the tiles
static int bwd_filter_slabs(const Geom& g, int c_in, int c_out) {
    const int mt = (c_in % 32 == 0) ? 2 : 1, nt = (c_out % 64 == 0) ? 4 : (c_out % 32 == 0 ? 2 : 1);
    return g.T * (c_in / (16 * mt)) * (c_out / (16 * nt));
}

int bwd_filter_chunks(const Geom& g, int c_in, int c_out, long long tiles_cap, bool mfma) {
    long long chunks;
    if (mfma) {
        const int slabs = bwd_filter_slabs(g, c_in, c_out);
        // all waves resident at once (two per SIMD), the same number of shares on every XCD
        chunks = (device_cu_count() * 8) / ((slabs + 3) / 4 * 4) / kXcds * kXcds;
        if (chunks < kXcds) chunks = kXcds;
        if (chunks > 256) chunks = 256;
    } else {
        const long long n_eb = ((long long)g.T * c_in * c_out + 255) / 256;
        chunks = (4096 + n_eb - 1) / n_eb;
        if (chunks > 512) chunks = 512;
    }
    if (chunks > tiles_cap) chunks = tiles_cap;
    if (chunks < 1) chunks = 1;
    return (int)chunks;
}

hipError_t launch_bwd_filter_mfma(const Geom& g, const float* x, int c_in, const float* gf, int c_out,
                                  const unsigned* pairs, const unsigned short* tap_first, const uint2* tile_hdr,
                                  const int* cand_start, const int* tile_start, const Counters* ctr, int n_chunks,
                                  double* fpart, hipStream_t s) {
    const int groups = (bwd_filter_slabs(g, c_in, c_out) + 3) / 4;
    const unsigned blocks = (unsigned)(kXcds * groups * ((n_chunks + kXcds - 1) / kXcds));
#define SCNN_BWD_CASE(MT_, NT_)                                                                                   \
    hipLaunchKernelGGL((k_bwd_filter_mfma<MT_, NT_>), dim3(blocks), dim3(256), 0, s, g.T, c_in, c_out, x, gf, pairs, \
                       tap_first, tile_hdr, cand_start, tile_start, g.batch, ctr, n_chunks, groups, fpart)
    if (c_in % 32 == 0) {
        if (c_out % 64 == 0) SCNN_BWD_CASE(2, 4); else if (c_out % 32 == 0) SCNN_BWD_CASE(2, 2); else SCNN_BWD_CASE(2, 1);
    } else {
        if (c_out % 64 == 0) SCNN_BWD_CASE(1, 4); else if (c_out % 32 == 0) SCNN_BWD_CASE(1, 2); else SCNN_BWD_CASE(1, 1);
    }
#undef SCNN_BWD_CASE
    return hipGetLastError();
}

// ------------------------------------------------------------------ bp_filter: add the partials, mask, round
// Eq. 3, second line: a weight that is exactly zero (pruned) receives no gradient.
__global__ __launch_bounds__(256) void k_bwd_filter_finish(const double* __restrict__ fpart, int n_chunks,
                                                           long long n_elem, const float* __restrict__ w,
                                                           float* __restrict__ bp_filter) {
    // 64 elements per workgroup; four threads per element each add a quarter of the partials (ascending), then
    // the quarters are added in ascending order: the order of the additions never depends on timing
    __shared__ double s_q[4][64];
    const int el = threadIdx.x & 63, q = threadIdx.x >> 6;
    const long long e = (long long)blockIdx.x * 64 + el;
    double sum = 0.0;
    const bool live = e < n_elem && w[e] != 0.0f;
    if (live) {
        const int c0 = (int)((long long)q * n_chunks / 4), c1 = (int)((long long)(q + 1) * n_chunks / 4);
        for (int c = c0; c < c1; ++c) sum += fpart[(size_t)c * n_elem + e];
    }
    s_q[q][el] = sum;
    __syncthreads();
    if (q == 0 && e < n_elem) bp_filter[e] = (float)(((s_q[0][el] + s_q[1][el]) + s_q[2][el]) + s_q[3][el]);
}

// also the place where the call's status words are written: {input rows, gradient rows, flags, 0}
__global__ void k_bwd_status(const Counters* __restrict__ ctr, long long nnz_in, long long g_rows,
                             long long* __restrict__ info) {
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        info[0] = nnz_in;
        info[1] = g_rows;
        info[2] = (long long)ctr->flags;
        info[3] = 0;
    }
}

hipError_t launch_bwd_filter_finish(const double* fpart, int n_chunks, long long n_elem, const float* w,
                                    float* bp_filter, const Counters* ctr, long long nnz_in, long long g_rows,
                                    long long* info, hipStream_t s) {
    hipLaunchKernelGGL(k_bwd_filter_finish, dim3((unsigned)((n_elem + 63) / 64)), dim3(256), 0, s, fpart, n_chunks,
                       n_elem, w, bp_filter);
    hipLaunchKernelGGL(k_bwd_status, dim3(1), dim3(64), 0, s, ctr, nnz_in, g_rows, info);
    return hipGetLastError();
}

}  // namespace scnn
