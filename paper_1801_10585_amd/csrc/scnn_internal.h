// Internal declarations shared by the HIP translation units of libscnn.
// gfx950 only: 64-wide wavefronts, 64-bit ballots, 64-bit occupancy words.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/scnn.h"

namespace scnn {

constexpr int kTileRows = 128;    // candidate sites per response tile
constexpr int kHistBins = 2048;   // bins per radix-select pass (11-bit digits)
constexpr int kScanChunk = 2048;  // elements per block in the device scan
// matrix-core pair lists: pair = (local row of the tile << 24) | row of the other operand
constexpr unsigned kPairRowShift = 24;
constexpr unsigned kPairInMask = (1u << kPairRowShift) - 1u;

// Grid geometry, passed by value to kernels.
struct Geom {
    int ndim;
    int batch;
    int E[3];          // extent, unused axes = 1 (axis order: c_1 slowest .. c_ndim fastest)
    int K[3];          // filter size per axis, unused = 1
    int H[3];          // (K-1)/2
    int T;             // taps = prod(K)
    long long N;       // sites per sample
    long long Npad;    // N rounded up to a multiple of 64
    int Wps;           // 64-bit occupancy words per sample = Npad / 64
};

// One per (sample, channel) column of the response matrix.
struct ColState {
    unsigned tau;       // threshold key: the k-th strongest key of the column
    unsigned cut;       // entries equal to tau survive up to this position in the column (0xffffffff: all of them)
    unsigned n_eq;      // entries whose key equals tau
    unsigned q;         // how many of those survive (lowest lin first)
    unsigned tau_lo;    // bracket expected to hold tau, from a sample of the column: keys in [tau_lo, tau_hi] go to the
    unsigned tau_hi;    //   side buffer, keys above tau_hi are only counted
    unsigned n_nz;      // non-zero entries in the column
    unsigned n_above;   // entries above the bracket
    unsigned side_fill; // side-buffer entries written so far
    int done;           // 1 = tau and cut are final
    unsigned long long side_off;  // first side-buffer entry of the column
};

constexpr int kTicketStride = 32;  // 32-bit words between two ticket counters
// Accelerator dies (XCDs) of the part the tile orders are laid out for: MI355X has eight, each with its own L2, and
// deals the workgroups of a launch out to them in turn (workgroup i runs on XCD i % kXcds).  On a part that is
// partitioned differently the orders are still correct, the spans just stop matching the L2s.
constexpr int kXcds = 8;

// Device-resident counters produced on the way.
struct Counters {
    long long n_cand;     // candidate sites
    long long n_tiles;    // response tiles (each sample padded to a multiple of kTileRows)
    long long n_rows;     // rows after selection / ReLU
    long long n_pool;     // rows after pooling
    unsigned flags;       // SCNN_FLAG_*
    int any_tie;          // some column needs tie ranks
    unsigned finished;    // workgroups of the compaction pass that have ended
    unsigned ticket;      // next tile of the compaction pass
    unsigned bracket_failed;  // some column's threshold lay outside its sampled bracket
    unsigned cols_done;       // columns whose selection has ended
    // tiles handed out so far in each of the contraction kernels' tile spans (one per XCD); one counter per 128-byte line:
    // read-modify-writes on one line are served one after the other, whichever word they address
    // (two sets: the quad kernel runs once per group of 64 output channels, up to two groups)
    unsigned conv_ticket[2 * kXcds * kTicketStride];
};

__host__ __device__ inline long long round_up(long long x, long long m) { return (x + m - 1) / m * m; }

// Compute units of the current device (asked once per device; 256, the part the launch shapes were tuned on, if the
// runtime will not say).  The persistent kernels size their grids from it.
int device_cu_count();

__device__ inline long long lin_of(const Geom& g, int c0, int c1, int c2) {
    // unused leading axes have extent 1 and coordinate 0
    return ((long long)c0 * g.E[1] + c1) * g.E[2] + c2;
}

__device__ inline void site_of(const Geom& g, long long lin, int& c0, int& c1, int& c2) {
    c2 = (int)(lin % g.E[2]);
    lin /= g.E[2];
    c1 = (int)(lin % g.E[1]);
    c0 = (int)(lin / g.E[1]);
}
// The same for a site index inside one sample, which fits 32 bits (the candidate lists hold these): two 32-bit
// divisions instead of two 64-bit ones, which cost several times as many instructions.
__device__ inline void site_of(const Geom& g, unsigned lin, int& c0, int& c1, int& c2) {
    const unsigned e2 = (unsigned)g.E[2], e1 = (unsigned)g.E[1];
    const unsigned q = lin / e2;
    c2 = (int)(lin - q * e2);
    const unsigned q1 = q / e1;
    c1 = (int)(q - q1 * e1);
    c0 = (int)q1;
}

// coords rows are (b, c_1..c_ndim); internally sites always use three axes with
// the real axes right-aligned (2-D: axis 0 has extent 1).
__device__ inline void load_site(const Geom& g, const int32_t* row, int& b, int& c0, int& c1, int& c2) {
    b = row[0];
    if (g.ndim == 3) {
        c0 = row[1]; c1 = row[2]; c2 = row[3];
    } else {
        c0 = 0; c1 = row[1]; c2 = row[2];
    }
}

__device__ inline void store_site(const Geom& g, int32_t* row, int b, int c0, int c1, int c2) {
    row[0] = b;
    if (g.ndim == 3) {
        row[1] = c0; row[2] = c1; row[3] = c2;
    } else {
        row[1] = c1; row[2] = c2;
    }
}

__device__ inline bool site_in_grid(const Geom& g, int b, int c0, int c1, int c2) {
    return (unsigned)b < (unsigned)g.batch && (unsigned)c0 < (unsigned)g.E[0] && (unsigned)c1 < (unsigned)g.E[1] &&
           (unsigned)c2 < (unsigned)g.E[2];
}

// Order-preserving key of a response: larger key = stronger response.
// 0 is reserved for "not an entry".
__device__ inline unsigned score_key(float v, int mode) {
    unsigned u = __float_as_uint(v);
    if ((u & 0x7fffffffu) == 0u) return 0u;
    if (mode == SCNN_TOPK_ABS) return u & 0x7fffffffu;
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Locate the sample of a tile: tile_start[b] <= tile < tile_start[b+1].
__device__ inline int sample_of_tile(const int* tile_start, int batch, int tile) {
    int lo = 0, hi = batch - 1;
    while (lo < hi) {
        int mid = (lo + hi + 1) >> 1;
        if (tile_start[mid] <= tile) lo = mid; else hi = mid - 1;
    }
    return lo;
}

// Row index of the occupied site (b, c0, c1, c2), or -1: the inverse of get_update_id.
__device__ inline int lookup_row(const Geom& g, const unsigned long long* __restrict__ occ,
                                 const unsigned* __restrict__ occ_prefix, long long nnz_in, int b, int c0, int c1,
                                 int c2) {
    if (!site_in_grid(g, b, c0, c1, c2)) return -1;
    const long long key = (long long)b * g.Npad + lin_of(g, c0, c1, c2);
    const unsigned long long word = occ[key >> 6];
    const int bit = (int)(key & 63);
    if (!((word >> bit) & 1ull)) return -1;
    const long long row = (long long)occ_prefix[key >> 6] + __popcll(word & ((1ull << bit) - 1ull));
    return row < nnz_in ? (int)row : -1;  // only an unsorted input can trip this guard
}

// Neighbour rows of one site along one filter line: the taps (t0, t1, t2_lo .. t2_lo + count - 1), count <= 32, look
// at the sites (c0 + t0 - H0, c1 + t1 - H1, c2 + t2 - H2), which are adjacent along the last axis and therefore sit
// in at most two adjacent 64-bit words of the occupancy bitmap.  Both words and their prefixes are loaded once and
// every tap of the line is resolved from them: emit(k, row) is called for k = 0 .. count-1 with the neighbour's row
// or -1.  `live` = false (a padding lane) emits -1 everywhere without touching memory contents that matter.
// 32-bit arithmetic throughout: site indices and bitmap word indices fit 31 bits.
template <typename Emit>
__device__ inline void lookup_line(const Geom& g, const unsigned long long* __restrict__ occ,
                                   const unsigned* __restrict__ occ_prefix, long long nnz_in, bool live, int b, int c0,
                                   int c1, int c2, int t0, int t1, int t2_lo, int count,
                                   const int* __restrict__ tap_active_line /* [t2_lo + k] */, Emit&& emit) {
    const int q0 = c0 + t0 - g.H[0], q1 = c1 + t1 - g.H[1];
    const bool line_ok = live && (unsigned)b < (unsigned)g.batch && (unsigned)q0 < (unsigned)g.E[0] &&
                         (unsigned)q1 < (unsigned)g.E[1];
    const int q2s = c2 + t2_lo - g.H[2];               // site of tap k is q2s + k
    const int k_lo = q2s < 0 ? -q2s : 0;               // first tap whose site is on the line
    const unsigned line_bit0 = (unsigned)((q0 * g.E[1] + q1) * g.E[2]);  // site index of (q0, q1, 0), if line_ok
    const unsigned first_bit = line_ok ? line_bit0 + (unsigned)(q2s + k_lo) : 0u;
    const unsigned w_rel = first_bit >> 6;             // word of the sample holding the first looked-at site
    const unsigned w0 = (unsigned)b * (unsigned)g.Wps + w_rel;
    const unsigned w_last = (unsigned)g.batch * (unsigned)g.Wps - 1u;
    const unsigned wa = line_ok ? (w0 < w_last ? w0 : w_last) : 0u, wb = wa < w_last ? wa + 1u : wa;
    const unsigned long long word_a = occ[wa], word_b = occ[wb];
    const unsigned pre_a = occ_prefix[wa], pre_b = occ_prefix[wb];
    for (int k = 0; k < count; ++k) {
        int n = -1;
        const int q2 = q2s + k;
        if (line_ok && (unsigned)q2 < (unsigned)g.E[2] && tap_active_line[k] != 0) {
            const unsigned bitpos = line_bit0 + (unsigned)q2;
            const bool second = (bitpos >> 6) != w_rel;
            const unsigned long long word = second ? word_b : word_a;
            const unsigned bit = bitpos & 63u;
            if ((word >> bit) & 1ull) {
                const long long rr = (long long)(second ? pre_b : pre_a) + __popcll(word & ((1ull << bit) - 1ull));
                if (rr < nnz_in) n = (int)rr;  // only an unsorted input can trip this guard
            }
        }
        emit(k, n);
    }
}

// Bits destined for a bitmap, one (word index, bits) per lane, where lanes that address the same word sit next to
// each other (rows sorted by site): OR the bits of each run of equal words into its first lane and report whether
// this lane is such a first lane.  Lanes with nothing to contribute pass a word index no other lane uses (negative).
// Every lane of the wave must call it.
__device__ inline bool wave_or_runs(long long word, unsigned long long& bits) {
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const long long ow = __shfl_down(word, d, 64);
        const unsigned long long ob = __shfl_down(bits, d, 64);
        if (lane + d < 64 && ow == word) bits |= ob;
    }
    const long long pw = __shfl_up(word, 1, 64);
    return lane == 0 || pw != word;
}

// Exclusive scan across a 256-thread block; `total` receives the block sum.
// Contains __syncthreads(): every thread of the block must call it.
__device__ inline unsigned block_exclusive_scan_256(unsigned v, unsigned* s_wave /*[4], shared*/, unsigned& total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    unsigned inc = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        unsigned t = __shfl_up(inc, d, 64);
        if (lane >= d) inc += t;
    }
    if (lane == 63) s_wave[wave] = inc;
    __syncthreads();
    unsigned base = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        unsigned x = s_wave[w];
        if (w < wave) base += x;
        tot += x;
    }
    total = tot;
    __syncthreads();
    return base + inc - v;
}

// Per-sample tile ranges and 16-row group ranges from the per-sample candidate ranges (cand_start[0 .. batch], in
// global memory and visible to the block): tile_start[b] = tiles of all earlier samples, each sample rounded up to
// whole tiles; rows16_start likewise in groups of 16 rows.  Either output may be null.  Returns the number of tiles.
// A scan over the samples, 256 at a time, so that batches of thousands of small samples cost a few rounds rather
// than one thread's walk over all of them.  Contains __syncthreads(): whole block of 256 threads.
__device__ inline int sample_ranges_256(int batch, const int* cand_start, int* tile_start, int* rows16_start,
                                        unsigned* s_wave /*[4], shared*/) {
    unsigned carry_t = 0, carry_r = 0;
    for (int b0 = 0; b0 < batch; b0 += 256) {
        const int b = b0 + (int)threadIdx.x;
        const int n = b < batch ? cand_start[b + 1] - cand_start[b] : 0;
        const unsigned t = (unsigned)((n + kTileRows - 1) / kTileRows), r = (unsigned)((n + 15) / 16);
        unsigned tot_t, tot_r;
        const unsigned et = block_exclusive_scan_256(t, s_wave, tot_t);
        const unsigned er = block_exclusive_scan_256(r, s_wave, tot_r);
        if (b < batch) {
            if (tile_start) tile_start[b] = (int)(carry_t + et);
            if (rows16_start) rows16_start[b] = (int)(carry_r + er);
        }
        carry_t += tot_t;
        carry_r += tot_r;
    }
    if (threadIdx.x == 0) {
        if (tile_start) tile_start[batch] = (int)carry_t;
        if (rows16_start) rows16_start[batch] = (int)carry_r;
    }
    return (int)carry_t;
}

// ---- host-side launchers (one per kernel family), all asynchronous on `s` ----
struct ScanBufs {
    unsigned* block_sums;  // ceil(capacity / kScanChunk) + 1 entries
};

// fill `words` 32-bit words with zero
hipError_t launch_zero(void* p, size_t bytes, hipStream_t s);
hipError_t launch_calibration_copy(void* dst, const void* src, size_t bytes, hipStream_t s);

// In-place exclusive scan of vals[0..n) (n read from *n_dev if n_dev != nullptr, else n_imm; n <= capacity).
// total (if non-null) receives the sum as long long.
hipError_t launch_exclusive_scan(unsigned* vals, long long capacity, long long n_imm, const long long* n_dev,
                                 unsigned* block_sums, long long* total, hipStream_t s);

}  // namespace scnn

// ---------------------------------------------------------------------------
// Launchers implemented in the individual .hip files.
// A count that lives on the device is passed as (n_imm, n_dev): n_dev wins
// when non-null.
// ---------------------------------------------------------------------------
namespace scnn {

// scnn_index.hip
hipError_t launch_index_build(const Geom& g, const int32_t* coords, long long n_imm, const long long* n_dev,
                              long long n_cap, unsigned long long* occ, unsigned* occ_prefix, Counters* ctr,
                              hipStream_t s);
// wp / wb / wq: the filter in the layout of the vector / pair-list matrix-core / quad matrix-core kernel (exactly the
// one that will run is non-null)
hipError_t launch_prepare(const Geom& g, const float* w, int c_in, int c_out, int adjoint, int c_out_pad, double* wp,
                          float* wb, float* wq, int* tap_active, int* tap_coord, void* zero_p, size_t zero_bytes,
                          hipStream_t s);
// chunk_sums: null, or (for more than kEmitSmallWords and at most kEmitMidWords words) counters that receive the
// candidate counts of chunks of 16 words (up to 32768 words) or 256 words (beyond), for launch_cand_emit_mid
hipError_t launch_cand_dilate(const Geom& g, const unsigned long long* occ, const int* tap_active,
                              unsigned long long* cand, unsigned* cand_count, unsigned* chunk_sums, hipStream_t s);
hipError_t launch_popcount(const unsigned long long* bits, long long n_words, unsigned* out, hipStream_t s);
// bitmaps of at most this many words: the emit kernels find their offsets themselves, no scan launch
constexpr long long kEmitSmallWords = 8192;
hipError_t launch_cand_emit_small(const Geom& g, const unsigned long long* cand, const unsigned* cand_count,
                                  long long n_words, unsigned* cand_lin, long long cand_cap, int* cand_start,
                                  int* tile_start, int* rows16_start, Counters* ctr, hipStream_t s);
// up to this many words the candidate list is emitted from per-chunk counts (8192 chunks of 256 words), no scan launch
constexpr int kEmitMidChunks = 8192;
constexpr long long kEmitMidWords = (long long)kEmitMidChunks * 256;
// Lanes that share a bitmap word in the candidate dilation: 16 on small grids, where one lane per word would leave
// most of the chip idle behind a chain of dependent loads (below about half a wave per SIMD), 1 on large grids.  A
// chunk, whose candidates the dilation counts, is what one workgroup of 256 threads covers per step: 16 or 256 words.
// Batches of many small samples (fewer than 256 words each) also take 16, as long as the chunk counts fit: a sample
// then starts at most 15 words into a chunk, and those are the words the emit kernel has to add up per sample.
inline int cand_dilate_lanes(long long n_words, long long words_per_sample) {
    return (n_words <= 32768 || (words_per_sample < 256 && n_words <= 16ll * kEmitMidChunks)) ? 16 : 1;
}
inline int cand_chunk_shift(long long n_words, long long words_per_sample) {
    return cand_dilate_lanes(n_words, words_per_sample) == 16 ? 4 : 8;
}
inline long long cand_chunk_count(long long n_words, long long words_per_sample) {
    const int sh = cand_chunk_shift(n_words, words_per_sample);
    return (n_words + (1ll << sh) - 1) >> sh;
}
hipError_t launch_cand_emit_mid(const Geom& g, const unsigned long long* cand, const unsigned* cand_count,
                                const unsigned* chunk_sums, long long n_words, unsigned* cand_lin, long long cand_cap,
                                int* cand_start, int* tile_start, int* rows16_start, Counters* ctr, hipStream_t s);
hipError_t launch_cand_emit(const Geom& g, const unsigned long long* cand, const unsigned* cand_prefix,
                            long long n_words, unsigned* cand_lin, long long cand_cap, int* cand_start,
                            int* tile_start, int* rows16_start, Counters* ctr, hipStream_t s);

// scnn_conv.hip
hipError_t launch_conv_valu(const Geom& g, const unsigned long long* occ, const unsigned* occ_prefix,
                            long long nnz_in, const float* feats, int c_in, const double* wp, int c_out,
                            int c_out_pad, const float* bias, const int* tap_active, const unsigned* cand_lin,
                            const int* cand_start, const int* tile_start, const Counters* ctr, long long tiles_cap,
                            float* resp, hipStream_t s);

bool conv_mfma_supported(const Geom& g, int c_in, int c_out, long long nnz_in);
hipError_t launch_pair_build(const Geom& g, const unsigned long long* occ, const unsigned* occ_prefix,
                             long long nnz_in, const int* tap_active, const int* tap_coord,
                             const unsigned* cand_lin, const int* cand_start, const int* tile_start,
                             const int* rows16_start, Counters* ctr, unsigned* pairs, unsigned short* block_tap,
                             uint2* tile_hdr, long long block_cap, long long tiles_cap,
                             unsigned short* tap_first /* nullable: [tiles][T + 1] first block of each tap */,
                             hipStream_t s);
hipError_t launch_conv_mfma(const Geom& g, long long nnz_in, const float* feats, int c_in, const float* wb, int c_out,
                            const float* bias, const unsigned* pairs, const unsigned short* block_tap,
                            const uint2* tile_hdr, Counters* ctr, float* resp, hipStream_t s);

// scnn_conv_quad.hip
constexpr int kQuadMaxCout = 128;  // two groups of 64 output channels, one launch each
// floats of the quad kernel's filter per group of 64 output channels: [tap][32-channel chunk][2048]
__host__ __device__ inline size_t quad_filter_floats(int taps, int c_in) { return (size_t)taps * ((c_in + 31) / 32) * 2048; }
inline int quad_groups(int c_out) { return (c_out + 63) / 64; }
bool conv_quad_supported(const Geom& g, int c_in, int c_out, long long nnz_in);
hipError_t launch_conv_quad(const Geom& g, const unsigned long long* occ, const unsigned* occ_prefix, long long nnz_in,
                            const float* feats, int c_in, const float* wq, int c_out, const float* bias,
                            const int* tap_active, const unsigned* cand_lin, const int* cand_start,
                            const int* tile_start, Counters* ctr, float* resp, int cus, hipStream_t s);

// scnn_bwd.hip
hipError_t launch_bwd_sites(const Geom& g, const int32_t* coords, long long rows, const int* cand_start,
                            unsigned* cand_lin, int* rows16_start, Counters* ctr, hipStream_t s);
hipError_t launch_bwd_data_write(const Geom& g, const float* resp, const float* x, int c_in, const int* cand_start,
                                 const int* tile_start, const Counters* ctr, long long tiles_cap, float* bp_data,
                                 hipStream_t s);
bool bwd_filter_mfma_supported(int c_in, int c_out, long long g_rows);
int bwd_filter_chunks(const Geom& g, int c_in, int c_out, long long tiles_cap, bool mfma);
hipError_t launch_bwd_filter_valu(const Geom& g, const unsigned long long* occ, const unsigned* occ_prefix,
                                  long long g_rows, const float* gf, int c_out, const float* x, int c_in,
                                  const int* tap_active, const unsigned* cand_lin, const int* cand_start,
                                  const int* tile_start, const Counters* ctr, int n_chunks, double* fpart,
                                  hipStream_t s);
hipError_t launch_bwd_filter_mfma(const Geom& g, const float* x, int c_in, const float* gf, int c_out,
                                  const unsigned* pairs, const unsigned short* tap_first, const uint2* tile_hdr,
                                  const int* cand_start, const int* tile_start, const Counters* ctr, int n_chunks,
                                  double* fpart, hipStream_t s);
hipError_t launch_bwd_filter_finish(const double* fpart, int n_chunks, long long n_elem, const float* w,
                                    float* bp_filter, const Counters* ctr, long long nnz_in, long long g_rows,
                                    long long* info, hipStream_t s);

// scnn_train.hip
hipError_t launch_density_regulariser(const float* feats, long long rows_imm, const long long* rows_dev,
                                      long long rows_cap, int channels, double n_total, double rho_up, double o,
                                      double b1, double b2, double lambda, const float* w, long long n_w, float* grad,
                                      unsigned long long* count, double* partial, double* out, hipStream_t s);
hipError_t launch_prune(float* w, unsigned char* warned, long long n, float eps, unsigned long long* counts,
                        hipStream_t s);

// scnn_topk.hip
hipError_t launch_rows_sample_bounds(const Geom& g, const int32_t* coords, long long rows, int* cand_start,
                                     int* tile_start, Counters* ctr, hipStream_t s);
hipError_t launch_rows_to_planar(const Geom& g, const int32_t* coords, const float* feats, int channels,
                                 const int* cand_start, const int* tile_start, const Counters* ctr,
                                 long long tiles_cap, unsigned* cand_lin, float* resp, hipStream_t s);
// Columns short enough for the one-workgroup selection (no sampled bracket, no marked rows).
bool topk_small_columns(const Geom& g);
// Row marks (all three nullable): row_keep, two 64-bit words per tile; row_plane, kMarkPlanes times as much;
// tile_base, one word per tile.  When given, the columns are not small and k > 0, tile_base[t] becomes the output row
// at which tile t starts, unless ctr->bracket_failed is set; launch_select_write must then be given tile_base.
constexpr int kTopkPartWords = 256;  // slices of a column at most
constexpr int kMarkPlanes = 64;  // one per channel where marks are used (up to 64 channels)
// Marks pay from 17 channels on: with fewer, few rows are marked by some channel's strong response and nearly every
// surviving entry of a bracket costs the settling pass an atomic.
constexpr int kMarkMinChannels = 16;
hipError_t launch_topk(const Geom& g, int channels, long long k, int mode, int relu, const int* tile_start,
                       const float* resp, ColState* cols, uint2* side,
                       uint2* part /* kTopkPartWords entries per column */, unsigned long long* row_keep,
                       unsigned long long* row_plane, long long* tile_base, long long tiles_cap, Counters* ctr,
                       hipStream_t s);
hipError_t launch_select_write(const Geom& g, int channels, int mode, int relu, const int* cand_start,
                               const int* tile_start, const unsigned* cand_lin, const float* resp,
                               const ColState* cols, unsigned long long* tile_state, long long tiles_cap,
                               Counters* ctr, int32_t* out_coords, float* out_feats, long long out_capacity,
                               long long* nnz_out /* nullable: also write the result counters */, long long aux_imm,
                               int aux_is_cand, const long long* tile_base /* nullable: from launch_topk */,
                               hipStream_t s);

// scnn_rows.hip
hipError_t launch_relu(const Geom& g, const int32_t* coords, const float* feats, long long rows, int channels,
                       unsigned* flags, unsigned* offs, unsigned* scan_block_sums, int32_t* out_coords, float* out_feats,
                       long long out_capacity, Counters* ctr, hipStream_t s);
hipError_t launch_maxpool(const Geom& g, const Geom& gp, const int32_t* coords, const float* feats,
                          long long n_imm, const long long* n_dev, long long n_cap, int channels,
                          int rows_have_entries, unsigned long long* occ, unsigned* occ_prefix, unsigned long long* pbits,
                          unsigned* pprefix, unsigned* scan_block_sums, long long* pool_key, long long pool_cap,
                          int32_t* out_coords, float* out_feats, long long out_capacity, Counters* ctr,
                          long long* nnz_out /* nullable: also write the result counters, as launch_finish would */,
                          long long aux_imm, int aux_is_cand, hipStream_t s);
hipError_t launch_to_dense(const Geom& g, const int32_t* coords, const float* feats, long long rows,
                           const long long* rows_dev, int channels, float* dense, hipStream_t s);
hipError_t launch_validate(const Geom& g, const int32_t* coords, long long rows, Counters* ctr, hipStream_t s);
hipError_t launch_finish(const Counters* ctr, int which_rows /*0 n_rows, 1 n_pool*/, long long aux_imm,
                         int aux_is_cand, long long out_capacity, long long* nnz_out, hipStream_t s);

}  // namespace scnn
