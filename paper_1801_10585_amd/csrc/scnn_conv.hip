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

// ---------------------------------------------------------------------------
// Matrix-core kernel for wide channels (C_in a multiple of 32, C_out a multiple
// of 16 up to 64): the gathered neighbour block of one tap really is a dense
// [pairs x C_in] . [C_in x C_out] contraction.
//
// Only about a third of a surface candidate's taps have a neighbour, and which
// ones varies from site to site, so zero-padding absent neighbours would waste
// most of the matrix cores.  Instead, per tile of 128 candidate sites and per
// tap, the present (output row, input row) pairs are packed into blocks of 16;
// each block is an fp32 MFMA chain per 32 input channels; its 16 x 16 results
// are added to the tile's accumulators in LDS.  Those accumulators are fp64
// (native LDS ds_add_f64): the fp32 matrix cores only ever sum 32 products of a
// single tap, the long cancelling sum over channels and taps is carried in
// double and rounded to fp32 once.
//
// Wave w of a workgroup owns output channels [16w, 16w+16) and walks every
// (tap, block) in ascending order, so each accumulator has a single writer and
// a fixed summation order: the result is bit-reproducible.
// ---------------------------------------------------------------------------
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kMfmaTapChunk = 32;                 // taps staged per stage (pair lists in LDS)
constexpr unsigned kPairRowShift = 24;            // pair = (local output row << 24) | input row
constexpr unsigned kPairInMask = (1u << kPairRowShift) - 1u;
constexpr unsigned kPadPair = (unsigned)kTileRows << kPairRowShift;  // list padding: dummy accumulator row, input row 0
constexpr int kMaxBlocks = kMfmaTapChunk * (kTileRows / 16);          // 16-pair blocks of one stage, at most

__host__ __device__ inline int conv_mfma_tap_chunk(int taps) { return taps < kMfmaTapChunk ? taps : kMfmaTapChunk; }

__host__ __device__ inline size_t conv_mfma_lds_bytes(int c_out, int taps) {
    return (size_t)(kTileRows + 1) * (c_out + 1) * sizeof(double)                  // accumulators + one dummy row
           + (size_t)conv_mfma_tap_chunk(taps) * kTileRows * sizeof(unsigned)       // packed pair list
           + (size_t)kTileRows * 3 * sizeof(short)                                  // candidate sites, later reused
                                                                                    // for the tap of each block
           + kMfmaTapChunk;                                                         // blocks per tap
}

// Operands of one group of GB consecutive 16-pair blocks, fetched one group ahead of their use.
template <int KC, int GB>
struct GroupRegs {
    f32x4 a[GB][KC][2];     // A operand: lane holds x[in(pair 16j + jj)][kc*32 + 8*gq .. + 8)
    float b[GB][KC][8];     // B operand: lane holds w[tap of block][kc*32 + 8*gq + s][16*wave + jj]
    unsigned oaddr[GB][4];  // LDS byte offset of the accumulator of result row 4*gq + v, this lane's channel
};

template <int KC /* C_in / 32 */, int NB /* C_out / 16 = waves per workgroup */>
__global__ __launch_bounds__(NB * 64) void k_conv_mfma(Geom g, const unsigned long long* __restrict__ occ,
                                                       const unsigned* __restrict__ occ_prefix, long long nnz_in,
                                                       const float* __restrict__ feats,
                                                       const float* __restrict__ w, const float* __restrict__ bias,
                                                       const int* __restrict__ tap_active,
                                                       const int* __restrict__ tap_coord,
                                                       const unsigned* __restrict__ cand_lin,
                                                       const int* __restrict__ cand_start,
                                                       const int* __restrict__ tile_start,
                                                       const Counters* __restrict__ ctr, float* __restrict__ resp) {
    constexpr int C_IN = KC * 32, C_OUT = NB * 16, CS = C_OUT + 1 /* padded accumulator row */;
    constexpr int GB = KC == 1 ? 4 : (KC == 2 ? 2 : 1);        // blocks per group
    constexpr int NT = NB * 64;
    constexpr int TPW = (kMfmaTapChunk + NB - 1) / NB;          // taps a wave looks up and packs per stage
    extern __shared__ __align__(16) unsigned char smem[];
    const int chunk = conv_mfma_tap_chunk(g.T);
    double* s_c = (double*)smem;                                             // [129][CS]; row 128 absorbs padding
    unsigned* s_flat = (unsigned*)(s_c + (kTileRows + 1) * CS);              // packed pairs, blocks of 16
    short* s_site = (short*)(s_flat + chunk * kTileRows);                    // [128][3], dead once read into registers
    unsigned char* s_btap = (unsigned char*)s_site;                          // [kMaxBlocks] tap of each block
    unsigned char* s_nblk = (unsigned char*)(s_site + kTileRows * 3);        // [32] blocks per tap
    static_assert(kMaxBlocks <= kTileRows * 3 * (int)sizeof(short), "block-tap table must fit the site table");

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int jj = lane & 15, gq = lane >> 4;
    const unsigned long long lt_mask = (1ull << lane) - 1ull;
    const int n_tiles = (int)ctr->n_tiles;
    const unsigned lane_off = (unsigned)(wave * 16 + jj) * (unsigned)sizeof(double);
    const unsigned in_max = (unsigned)(nnz_in - 1);

    // XCD-aware tile order: workgroup i runs on XCD i % 8; give each XCD one contiguous span of tiles so that
    // the input rows shared by neighbouring tiles stay in that XCD's L2.
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3, per_xcd = gridDim.x >> 3;
    const int span = (n_tiles + 7) >> 3;
    const int tile_end = (xcd + 1) * span < n_tiles ? (xcd + 1) * span : n_tiles;

    for (int tile = xcd * span + slot; tile < tile_end; tile += per_xcd) {
        const int b = sample_of_tile(tile_start, g.batch, tile);
        const int first = cand_start[b] + (tile - tile_start[b]) * kTileRows;
        int nrows = cand_start[b + 1] - first;
        if (nrows > kTileRows) nrows = kTileRows;

        __syncthreads();  // previous tile's epilogue has read the accumulators
        for (int r = threadIdx.x; r < kTileRows; r += NT) {
            int c0 = 0, c1 = 0, c2 = 0;
            if (r < nrows) site_of(g, cand_lin[first + r], c0, c1, c2);
            s_site[r * 3 + 0] = (short)c0;
            s_site[r * 3 + 1] = (short)c1;
            s_site[r * 3 + 2] = (short)c2;
        }
        for (int i = threadIdx.x; i < kTileRows * CS; i += NT) s_c[i] = 0.0;  // the dummy row needs no reset
        __syncthreads();
        int sc[2][3];  // sites of rows lane and lane + 64
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int a = 0; a < 3; ++a) sc[h][a] = s_site[(h * 64 + lane) * 3 + a];

        for (int tc = 0; tc < g.T; tc += chunk) {
            const int tmax = (g.T - tc) < chunk ? (g.T - tc) : chunk;
            __syncthreads();  // sites read; pair list of the previous stage consumed; accumulators zeroed
            // ---- neighbour lookup: wave handles taps wave, wave + NB, ... for rows lane and lane + 64.  All occupancy
            //      words are requested first, then all prefixes, so that the loads overlap.
            long long key[TPW][2];
            unsigned long long word[TPW][2];
            unsigned nbr[TPW][2];
#pragma unroll
            for (int m = 0; m < TPW; ++m) {
                const int tt = wave + m * NB;
                const bool live = tt < tmax && tap_active[tc + (tt < tmax ? tt : 0)];
                const int tc3 = tap_coord[tc + (tt < tmax ? tt : 0)];  // (t0, t1, t2) packed one byte each
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    key[m][h] = -1;
                    word[m][h] = 0;
                    const int q0 = sc[h][0] + (tc3 & 255) - g.H[0], q1 = sc[h][1] + ((tc3 >> 8) & 255) - g.H[1],
                              q2 = sc[h][2] + (tc3 >> 16) - g.H[2];
                    if (live && h * 64 + lane < nrows && site_in_grid(g, b, q0, q1, q2)) {
                        key[m][h] = (long long)b * g.Npad + lin_of(g, q0, q1, q2);
                        word[m][h] = occ[key[m][h] >> 6];
                    }
                }
            }
#pragma unroll
            for (int m = 0; m < TPW; ++m)
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    unsigned n = 0xffffffffu;
                    const int bit = (int)(key[m][h] & 63);
                    if (key[m][h] >= 0 && ((word[m][h] >> bit) & 1ull)) {
                        const long long row = (long long)occ_prefix[key[m][h] >> 6] +
                                              __popcll(word[m][h] & ((1ull << bit) - 1ull));
                        if (row < nnz_in) n = (unsigned)row;
                    }
                    nbr[m][h] = n;
                }
            // ---- blocks per tap
#pragma unroll
            for (int m = 0; m < TPW; ++m) {
                const int tt = wave + m * NB;
                const int cnt = __popcll(__ballot(nbr[m][0] != 0xffffffffu)) + __popcll(__ballot(nbr[m][1] != 0xffffffffu));
                if (lane == 0 && tt < kMfmaTapChunk) s_nblk[tt] = (unsigned char)((cnt + 15) >> 4);
            }
            __syncthreads();
            // ---- pack: taps in ascending order, each tap's present pairs in ascending output row, padded to whole
            //      blocks of 16 with entries that point at the dummy accumulator row
            int blk_incl = lane < tmax ? (int)s_nblk[lane] : 0;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const int t = __shfl_up(blk_incl, d, 64);
                if (lane >= d) blk_incl += t;
            }
            const int n_blocks = __shfl(blk_incl, 63, 64);
#pragma unroll
            for (int m = 0; m < TPW; ++m) {
                const int tt = wave + m * NB;
                const int src = tt < 64 ? tt : 63;
                const int incl = __shfl(blk_incl, src, 64);
                const int nblk = tt < tmax ? (int)s_nblk[tt < kMfmaTapChunk ? tt : 0] : 0;
                const int blk0 = incl - nblk;
                unsigned* pl = s_flat + blk0 * 16;
                const unsigned long long m0 = __ballot(nbr[m][0] != 0xffffffffu), m1 = __ballot(nbr[m][1] != 0xffffffffu);
                const int c0 = __popcll(m0), cnt = c0 + __popcll(m1);
                if (nbr[m][0] != 0xffffffffu) pl[__popcll(m0 & lt_mask)] = ((unsigned)lane << kPairRowShift) | nbr[m][0];
                if (nbr[m][1] != 0xffffffffu)
                    pl[c0 + __popcll(m1 & lt_mask)] = ((unsigned)(64 + lane) << kPairRowShift) | nbr[m][1];
                if (cnt + lane < nblk * 16) pl[cnt + lane] = kPadPair;
                if (lane < nblk) s_btap[blk0 + lane] = (unsigned char)tt;
            }
            __syncthreads();

            // ---- contraction: this wave's 16 output channels, every block in ascending (tap, output row) order
            if (n_blocks > 0) {
                const int n_groups = (n_blocks + GB - 1) / GB;
                // All loads of a group are unconditional so that their number is fixed: a group past the end repeats
                // the last one, a block past the end reads whatever the list holds there (tap and input row are
                // clamped) and is never computed.
                auto load_group = [&](int gi, GroupRegs<KC, GB>& R) {
                    const int g0 = (gi < n_groups ? gi : n_groups - 1) * GB;
                    unsigned e_in[GB];
                    uint4 e_out[GB];
                    int tap[GB];
#pragma unroll
                    for (int k = 0; k < GB; ++k) {
                        e_in[k] = s_flat[16 * (g0 + k) + jj];
                        e_out[k] = *(const uint4*)(s_flat + 16 * (g0 + k) + 4 * gq);
                        tap[k] = s_btap[g0 + k];
                    }
#pragma unroll
                    for (int k = 0; k < GB; ++k) {
                        int tt = __builtin_amdgcn_readfirstlane(tap[k]);
                        tt = tt < tmax ? tt : tmax - 1;
                        const float* wt = w + ((size_t)(tc + tt) * C_IN) * C_OUT + wave * 16 + jj;
#pragma unroll
                        for (int kc = 0; kc < KC; ++kc)
#pragma unroll
                            for (int s = 0; s < 8; ++s) R.b[k][kc][s] = wt[(size_t)(kc * 32 + 8 * gq + s) * C_OUT];
                        unsigned in = e_in[k] & kPairInMask;
                        in = in < in_max ? in : in_max;
                        const f32x4* src = (const f32x4*)(feats + (size_t)in * C_IN + 8 * gq);
#pragma unroll
                        for (int kc = 0; kc < KC; ++kc) {
                            R.a[k][kc][0] = src[kc * 8];
                            R.a[k][kc][1] = src[kc * 8 + 1];
                        }
                        R.oaddr[k][0] = (e_out[k].x >> kPairRowShift) * (unsigned)(CS * sizeof(double)) + lane_off;
                        R.oaddr[k][1] = (e_out[k].y >> kPairRowShift) * (unsigned)(CS * sizeof(double)) + lane_off;
                        R.oaddr[k][2] = (e_out[k].z >> kPairRowShift) * (unsigned)(CS * sizeof(double)) + lane_off;
                        R.oaddr[k][3] = (e_out[k].w >> kPairRowShift) * (unsigned)(CS * sizeof(double)) + lane_off;
                    }
                };
                // NBK blocks as straight-line code: independent fp32 MFMA chains (one per block and per 32 input
                // channels), then the 16 x 16 results (rows = pairs 4*gq + v, column = channel 16*wave + jj) are added
                // to the fp64 accumulators.  Padding pairs land in the dummy row.
                auto compute_blocks = [&](auto nbk_tag, const GroupRegs<KC, GB>& R) {
                    constexpr int NBK = decltype(nbk_tag)::value;
                    f32x4 acc[NBK][KC];
#pragma unroll
                    for (int k = 0; k < NBK; ++k)
#pragma unroll
                        for (int kc = 0; kc < KC; ++kc) {
                            f32x4 c = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                            for (int s = 0; s < 4; ++s)
                                c = __builtin_amdgcn_mfma_f32_16x16x4f32(R.a[k][kc][0][s], R.b[k][kc][s], c, 0, 0, 0);
#pragma unroll
                            for (int s = 0; s < 4; ++s)
                                c = __builtin_amdgcn_mfma_f32_16x16x4f32(R.a[k][kc][1][s], R.b[k][kc][4 + s], c, 0, 0, 0);
                            acc[k][kc] = c;
                        }
#pragma unroll
                    for (int k = 0; k < NBK; ++k)
#pragma unroll
                        for (int kc = 0; kc < KC; ++kc)
#pragma unroll
                            for (int v = 0; v < 4; ++v)
                                __hip_atomic_fetch_add((double*)((unsigned char*)s_c + R.oaddr[k][v]),
                                                       (double)acc[k][kc][v], __ATOMIC_RELAXED,
                                                       __HIP_MEMORY_SCOPE_WORKGROUP);
                };
                auto compute_group = [&](int gi, const GroupRegs<KC, GB>& R) {
                    const int nb = n_blocks - gi * GB;  // >= 1
                    if (nb >= GB) {
                        compute_blocks(std::integral_constant<int, GB>{}, R);
                    } else if constexpr (GB >= 2) {
                        if (nb == 1) compute_blocks(std::integral_constant<int, 1>{}, R);
                        if constexpr (GB >= 4) {
                            if (nb == 2) compute_blocks(std::integral_constant<int, 2>{}, R);
                            if (nb == 3) compute_blocks(std::integral_constant<int, 3>{}, R);
                        }
                    }
                };
                GroupRegs<KC, GB> r0, r1;
                load_group(0, r0);
                for (int gi = 0; gi < n_groups; gi += 2) {
                    load_group(gi + 1, r1);
                    compute_group(gi, r0);
                    load_group(gi + 2, r0);
                    if (gi + 1 < n_groups) compute_group(gi + 1, r1);
                }
            }
        }
        __syncthreads();
        // ---- epilogue: one rounding to fp32, bias on the non-zero entries, planar store
        for (int i = threadIdx.x; i < kTileRows * C_OUT; i += NT) {
            const int r = i & (kTileRows - 1), oc = i >> 7;
            float v = (float)s_c[r * CS + oc];
            if (bias && v != 0.0f) v += bias[oc];
            resp[((size_t)tile * C_OUT + oc) * kTileRows + r] = v;
        }
    }
}

template <int KC, int NB>
static hipError_t launch_conv_mfma_t(const Geom& g, const unsigned long long* occ, const unsigned* occ_prefix,
                                     long long nnz_in, const float* feats, const float* w, const float* bias,
                                     const int* tap_active, const int* tap_coord, const unsigned* cand_lin,
                                     const int* cand_start, const int* tile_start, const Counters* ctr, float* resp,
                                     hipStream_t s) {
    const size_t lds = conv_mfma_lds_bytes(NB * 16, g.T);
    static size_t attr_lds = 0;
    if (attr_lds < lds) {
        hipError_t e = hipFuncSetAttribute((const void*)k_conv_mfma<KC, NB>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_lds = lds;
    }
    int per_cu = (int)((160 * 1024) / lds);
    if (per_cu < 1) per_cu = 1;
    if (per_cu * NB > 16) per_cu = 16 / NB;  // at most 16 waves per CU are useful here
    const int grid = 256 * per_cu;           // a multiple of 8 (one span of tiles per XCD)
    hipLaunchKernelGGL((k_conv_mfma<KC, NB>), dim3(grid), dim3(NB * 64), lds, s, g, occ, occ_prefix, nnz_in, feats, w,
                       bias, tap_active, tap_coord, cand_lin, cand_start, tile_start, ctr, resp);
    return hipGetLastError();
}

bool conv_mfma_supported(const Geom& g, int c_in, int c_out, long long nnz_in) {
    if (g.E[0] > 32767 || g.E[1] > 32767 || g.E[2] > 32767) return false;  // sites are staged as 16-bit coordinates
    return c_in % 32 == 0 && c_in <= 128 && c_out % 16 == 0 && c_out <= 64 && nnz_in > 0 &&
           nnz_in < (1ll << kPairRowShift);
}

hipError_t launch_conv_mfma(const Geom& g, const unsigned long long* occ, const unsigned* occ_prefix,
                            long long nnz_in, const float* feats, int c_in, const float* w, int c_out,
                            const float* bias, const int* tap_active, const int* tap_coord,
                            const unsigned* cand_lin, const int* cand_start, const int* tile_start,
                            const Counters* ctr, float* resp, hipStream_t s) {
#define SCNN_MFMA_CASE(KC_, NB_)                                                                                  \
    if (c_in == KC_ * 32 && c_out == NB_ * 16)                                                                    \
        return launch_conv_mfma_t<KC_, NB_>(g, occ, occ_prefix, nnz_in, feats, w, bias, tap_active, tap_coord,    \
                                            cand_lin, cand_start, tile_start, ctr, resp, s);
    SCNN_MFMA_CASE(1, 1) SCNN_MFMA_CASE(1, 2) SCNN_MFMA_CASE(1, 3) SCNN_MFMA_CASE(1, 4)
    SCNN_MFMA_CASE(2, 1) SCNN_MFMA_CASE(2, 2) SCNN_MFMA_CASE(2, 3) SCNN_MFMA_CASE(2, 4)
    SCNN_MFMA_CASE(3, 1) SCNN_MFMA_CASE(3, 2) SCNN_MFMA_CASE(3, 3) SCNN_MFMA_CASE(3, 4)
    SCNN_MFMA_CASE(4, 1) SCNN_MFMA_CASE(4, 2) SCNN_MFMA_CASE(4, 3) SCNN_MFMA_CASE(4, 4)
#undef SCNN_MFMA_CASE
    return hipErrorInvalidValue;
}

}  // namespace scnn
