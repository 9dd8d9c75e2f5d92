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
constexpr int kMaxRounds = 8 * kMfmaTapChunk;     // >= sum over a stage's taps of ceil(blocks / RB), RB >= 1

__host__ __device__ inline int conv_mfma_tap_chunk(int taps) { return taps < kMfmaTapChunk ? taps : kMfmaTapChunk; }

__host__ __device__ inline size_t conv_mfma_lds_bytes(int c_out, int taps) {
    return (size_t)kTileRows * (c_out + 1) * sizeof(double)                        // accumulators
           + (size_t)conv_mfma_tap_chunk(taps) * kTileRows * sizeof(unsigned)       // pair lists
           + kMfmaTapChunk * sizeof(int)                                            // pair counts
           + (size_t)kTileRows * 3 * sizeof(short)                                  // candidate sites
           + (size_t)kMaxRounds * sizeof(unsigned short) + 16;                      // round list + its length
}

// One "round" = up to RB consecutive 16-pair blocks of one tap.  Its operands are fetched one round ahead of
// their use (fixed number of loads per round, so the hardware wait counters can be set exactly).
template <int KC, int RB>
struct RoundRegs {
    f32x4 a[RB][KC][2];   // A operand: lane holds x[in(pair 16j + jj)][kc*32 + 8*gq .. + 8)
    float b[KC][8];       // B operand: lane holds w[t][kc*32 + 8*gq + s][16*wave + jj]
    int orow[RB][4];      // output rows of result rows 4*gq + v (or -1)
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
    constexpr int RB = KC == 1 ? 4 : (KC == 2 ? 2 : 1);
    constexpr int NT = NB * 64;
    extern __shared__ __align__(16) unsigned char smem[];
    const int chunk = conv_mfma_tap_chunk(g.T);
    double* s_c = (double*)smem;                                             // [128][CS]
    unsigned* s_pair = (unsigned*)(s_c + kTileRows * CS);                    // [chunk][128]
    int* s_cnt = (int*)(s_pair + chunk * kTileRows);                         // [32]
    short* s_site = (short*)(s_cnt + kMfmaTapChunk);                         // [128][3]
    unsigned short* s_round = (unsigned short*)(s_site + kTileRows * 3);     // [kMaxRounds]: tap | j0 << 5 | nb << 9
    int* s_nrounds = (int*)(s_round + kMaxRounds);

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int jj = lane & 15, gq = lane >> 4;
    const unsigned long long lt_mask = (1ull << lane) - 1ull;
    const int n_tiles = (int)ctr->n_tiles;

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
        for (int i = threadIdx.x; i < kTileRows * CS; i += NT) s_c[i] = 0.0;

        for (int tc = 0; tc < g.T; tc += chunk) {
            const int tmax = (g.T - tc) < chunk ? (g.T - tc) : chunk;
            __syncthreads();  // sites written; pair lists of the previous stage consumed; accumulators zeroed
            // ---- neighbour lookup, all (tap, row) items independent so that many loads are in flight
            for (int base = 0; base < tmax * kTileRows; base += NT * 8) {
                long long key[8];
                unsigned long long word[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int idx = base + u * NT + threadIdx.x;
                    const int tt = idx >> 7, r = idx & (kTileRows - 1);
                    key[u] = -1;
                    word[u] = 0;
                    if (idx < tmax * kTileRows && r < nrows && tap_active[tc + tt]) {
                        const int tc3 = tap_coord[tc + tt];  // (t0, t1, t2) packed one byte each
                        const int q0 = s_site[r * 3 + 0] + (tc3 & 255) - g.H[0],
                                  q1 = s_site[r * 3 + 1] + ((tc3 >> 8) & 255) - g.H[1],
                                  q2 = s_site[r * 3 + 2] + (tc3 >> 16) - g.H[2];
                        if (site_in_grid(g, b, q0, q1, q2)) {
                            key[u] = (long long)b * g.Npad + lin_of(g, q0, q1, q2);
                            word[u] = occ[key[u] >> 6];
                        }
                    }
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int idx = base + u * NT + threadIdx.x;
                    if (idx < tmax * kTileRows) {
                        unsigned n = 0xffffffffu;
                        const int bit = (int)(key[u] & 63);
                        if (key[u] >= 0 && ((word[u] >> bit) & 1ull)) {
                            const long long row =
                                (long long)occ_prefix[key[u] >> 6] + __popcll(word[u] & ((1ull << bit) - 1ull));
                            if (row < nnz_in) n = (unsigned)row;
                        }
                        s_pair[idx] = n;
                    }
                }
            }
            __syncthreads();
            // ---- pack each tap's present pairs to the front of its list (in place, ascending output row)
            for (int tt = wave; tt < tmax; tt += NB) {
                unsigned* pl = s_pair + tt * kTileRows;
                const unsigned n0 = pl[lane], n1 = pl[64 + lane];
                const unsigned long long m0 = __ballot(n0 != 0xffffffffu), m1 = __ballot(n1 != 0xffffffffu);
                const int c0 = __popcll(m0);
                if (n0 != 0xffffffffu) pl[__popcll(m0 & lt_mask)] = ((unsigned)lane << kPairRowShift) | n0;
                if (n1 != 0xffffffffu)
                    pl[c0 + __popcll(m1 & lt_mask)] = ((unsigned)(64 + lane) << kPairRowShift) | n1;
                if (lane == 0) s_cnt[tt] = c0 + __popcll(m1);
            }
            __syncthreads();
            // ---- round list: (tap, first block, block count <= RB), taps ascending
            if (wave == 0) {
                int nr = 0, nblk = 0;
                if (lane < tmax) {
                    nblk = (s_cnt[lane] + 15) >> 4;
                    nr = (nblk + RB - 1) / RB;
                }
                int inc = nr;
#pragma unroll
                for (int d = 1; d < 64; d <<= 1) {
                    const int t = __shfl_up(inc, d, 64);
                    if (lane >= d) inc += t;
                }
                int o = inc - nr;
                for (int j0 = 0; j0 < nblk; j0 += RB, ++o) {
                    const int nb = (nblk - j0) < RB ? (nblk - j0) : RB;
                    s_round[o] = (unsigned short)(lane | (j0 << 5) | (nb << 9));
                }
                if (lane == 63) *s_nrounds = inc;
            }
            __syncthreads();

            // ---- contraction: this wave's 16 output channels, every round in ascending (tap, block) order
            const int n_rounds = __builtin_amdgcn_readfirstlane(*s_nrounds);
            if (n_rounds > 0) {
                auto load_round = [&](int i, RoundRegs<KC, RB>& R) {
                    const unsigned rd = s_round[i < n_rounds ? i : n_rounds - 1];  // clamped: loads are unconditional
                    const int tt = rd & 31, j0 = (rd >> 5) & 15, nb = rd >> 9;
                    const int n_t = s_cnt[tt];
                    const unsigned* pl = s_pair + tt * kTileRows;
                    const float* wt = w + ((size_t)(tc + tt) * C_IN) * C_OUT + wave * 16 + jj;
#pragma unroll
                    for (int kc = 0; kc < KC; ++kc)
#pragma unroll
                        for (int s = 0; s < 8; ++s) R.b[kc][s] = wt[(size_t)(kc * 32 + 8 * gq + s) * C_OUT];
                    // every LDS read below is unconditional (clamped index) so that they issue back to back
                    unsigned e_in[RB];
                    uint4 e_out[RB];
#pragma unroll
                    for (int k = 0; k < RB; ++k) {
                        const int p = 16 * (j0 + k) + jj, pv = 16 * (j0 + k) + 4 * gq;
                        e_in[k] = pl[p < kTileRows ? p : kTileRows - 1];
                        e_out[k] = *(const uint4*)(pl + (pv < kTileRows ? pv : kTileRows - 4));
                    }
#pragma unroll
                    for (int k = 0; k < RB; ++k) {
                        const int p = 16 * (j0 + k) + jj, pv = 16 * (j0 + k) + 4 * gq;
                        // pairs beyond the list read input row 0: their results are never stored
                        const unsigned in = (k < nb && p < n_t) ? (e_in[k] & kPairInMask) : 0u;
                        const f32x4* src = (const f32x4*)(feats + (size_t)in * C_IN + 8 * gq);
#pragma unroll
                        for (int kc = 0; kc < KC; ++kc) {
                            R.a[k][kc][0] = src[kc * 8];
                            R.a[k][kc][1] = src[kc * 8 + 1];
                        }
                        const bool kv = k < nb;
                        R.orow[k][0] = (kv && pv + 0 < n_t) ? (int)(e_out[k].x >> kPairRowShift) : -1;
                        R.orow[k][1] = (kv && pv + 1 < n_t) ? (int)(e_out[k].y >> kPairRowShift) : -1;
                        R.orow[k][2] = (kv && pv + 2 < n_t) ? (int)(e_out[k].z >> kPairRowShift) : -1;
                        R.orow[k][3] = (kv && pv + 3 < n_t) ? (int)(e_out[k].w >> kPairRowShift) : -1;
                    }
                };
                auto compute_round = [&](int i, const RoundRegs<KC, RB>& R) {
                    const int nb = s_round[i] >> 9;
#pragma unroll
                    for (int k = 0; k < RB; ++k) {
                        if (k < nb) {
                            // one fp32 MFMA chain per 32 input channels; each chain's 16 x 16 result (rows = pairs
                            // 4*gq + v, column = channel 16*wave + jj) is added to the fp64 accumulators
#pragma unroll
                            for (int kc = 0; kc < KC; ++kc) {
                                f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                                for (int s = 0; s < 4; ++s)
                                    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(R.a[k][kc][0][s], R.b[kc][s], acc, 0, 0, 0);
#pragma unroll
                                for (int s = 0; s < 4; ++s)
                                    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(R.a[k][kc][1][s], R.b[kc][4 + s], acc, 0,
                                                                               0, 0);
#pragma unroll
                                for (int v = 0; v < 4; ++v)
                                    if (R.orow[k][v] >= 0)
                                        __hip_atomic_fetch_add(&s_c[R.orow[k][v] * CS + wave * 16 + jj], (double)acc[v],
                                                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                            }
                        }
                    }
                };
                RoundRegs<KC, RB> r0, r1;
                load_round(0, r0);
                for (int i = 0; i < n_rounds; i += 2) {
                    load_round(i + 1, r1);
                    compute_round(i, r0);
                    load_round(i + 2, r0);
                    if (i + 1 < n_rounds) compute_round(i + 1, r1);
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
