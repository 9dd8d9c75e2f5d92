// Index build, candidate-site generation and the small device-wide scan.
//
// Step "decompress indices" of Algorithm 1 becomes: mark every occupied site in
// a bitmap over (sample, lin) and remember, per 64-bit word, the row index of
// its first occupied site.  Rows are sorted by (b, lin), so the row of any
// occupied site is  prefix[word] + popcount(bits below it)  -- the inverse of
// get_update_id without a hash table and without an r^d value buffer.
//
// Candidate output sites (the sites Algorithm 1's dense buffer could become
// non-zero at) are the occupied sites dilated by the filter's non-zero taps;
// they are marked in a second bitmap, counted per word, scanned, and written
// out as a sorted list of per-sample site indices.
#include <atomic>

#include "scnn_internal.h"

namespace scnn {

int device_cu_count() {
    static std::atomic<int> cache[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 256;
    int n = (dev >= 0 && dev < 64) ? cache[dev].load(std::memory_order_relaxed) : 0;
    if (n <= 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) return 256;
        if (dev >= 0 && dev < 64) cache[dev].store(n, std::memory_order_relaxed);
    }
    return n;
}


// ------------------------------------------------------------------ zero fill
__global__ void k_zero(uint4* __restrict__ p, size_t n16) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n16; i += stride) p[i] = make_uint4(0, 0, 0, 0);
}

hipError_t launch_zero(void* p, size_t bytes, hipStream_t s) {
    size_t n16 = (bytes + 15) / 16;
    if (n16 == 0) return hipSuccess;
    int blocks = (int)((n16 + 255) / 256);
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(k_zero, dim3(blocks), dim3(256), 0, s, (uint4*)p, n16);
    return hipGetLastError();
}

// Plain streaming copy of a known size: the yardstick against which the memory-traffic counters of the
// other kernels are scaled.
__global__ void k_calibration_copy(uint4* __restrict__ dst, const uint4* __restrict__ src, size_t n16) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n16; i += stride) dst[i] = src[i];
}

hipError_t launch_calibration_copy(void* dst, const void* src, size_t bytes, hipStream_t s) {
    const size_t n16 = bytes / 16;
    if (n16 == 0) return hipSuccess;
    size_t blocks = (n16 + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    hipLaunchKernelGGL(k_calibration_copy, dim3((unsigned)blocks), dim3(256), 0, s, (uint4*)dst, (const uint4*)src, n16);
    return hipGetLastError();
}

// ------------------------------------------------------------------ scan
__global__ __launch_bounds__(256) void k_scan_local(unsigned* __restrict__ vals, long long n_imm,
                                                    const long long* __restrict__ n_dev,
                                                    unsigned* __restrict__ block_sums) {
    __shared__ unsigned s_wave[4];
    const long long n = n_dev ? *n_dev : n_imm;
    const long long base = (long long)blockIdx.x * kScanChunk + (long long)threadIdx.x * 8;
    unsigned v[8];
    unsigned sum = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        v[i] = (base + i < n) ? vals[base + i] : 0u;
        sum += v[i];
    }
    unsigned total;
    unsigned excl = block_exclusive_scan_256(sum, s_wave, total);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        if (base + i < n) vals[base + i] = excl;
        excl += v[i];
    }
    if (threadIdx.x == 0) block_sums[blockIdx.x] = total;
}

__global__ __launch_bounds__(256) void k_scan_top(unsigned* __restrict__ block_sums, long long n_blocks,
                                                  long long* __restrict__ total_out) {
    __shared__ unsigned s_wave[4];
    unsigned carry = 0;
    for (long long start = 0; start < n_blocks; start += 256) {
        long long i = start + threadIdx.x;
        unsigned v = (i < n_blocks) ? block_sums[i] : 0u;
        unsigned total;
        unsigned excl = block_exclusive_scan_256(v, s_wave, total);
        if (i < n_blocks) block_sums[i] = carry + excl;
        carry += total;
    }
    if (threadIdx.x == 0 && total_out) *total_out = (long long)carry;
}

__global__ __launch_bounds__(256) void k_scan_add(unsigned* __restrict__ vals, long long n_imm,
                                                  const long long* __restrict__ n_dev,
                                                  const unsigned* __restrict__ block_sums) {
    const long long n = n_dev ? *n_dev : n_imm;
    const long long base = (long long)blockIdx.x * kScanChunk + (long long)threadIdx.x * 8;
    const unsigned add = block_sums[blockIdx.x];
    if (add == 0) return;
#pragma unroll
    for (int i = 0; i < 8; ++i)
        if (base + i < n) vals[base + i] += add;
}

// The whole scan in one workgroup, for short arrays (small grids): one launch instead of three.
__global__ __launch_bounds__(256) void k_scan_small(unsigned* __restrict__ vals, long long n_imm,
                                                    const long long* __restrict__ n_dev,
                                                    long long* __restrict__ total_out) {
    __shared__ unsigned s_wave[4];
    const long long n = n_dev ? *n_dev : n_imm;
    unsigned carry = 0;
    for (long long start = 0; start < n; start += kScanChunk) {
        const long long base = start + (long long)threadIdx.x * 8;
        unsigned v[8];
        unsigned sum = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            v[i] = (base + i < n) ? vals[base + i] : 0u;
            sum += v[i];
        }
        unsigned total;
        unsigned excl = carry + block_exclusive_scan_256(sum, s_wave, total);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (base + i < n) vals[base + i] = excl;
            excl += v[i];
        }
        carry += total;
    }
    if (threadIdx.x == 0 && total_out) *total_out = (long long)carry;
}

// up to this many elements one workgroup scans alone: it takes about 2 us per chunk of 2048, three launches 13 us
constexpr long long kScanSmall = 4 * kScanChunk;

// Second and last step of the scan of up to kScanTwoStep chunks: a block adds up the sums of the chunks before its
// own by itself (a few thousand numbers at most) instead of waiting for a launch that scans them.
constexpr long long kScanTwoStep = 4096;
__global__ __launch_bounds__(256) void k_scan_add_own(unsigned* __restrict__ vals, long long n_imm,
                                                      const long long* __restrict__ n_dev,
                                                      const unsigned* __restrict__ block_sums,
                                                      long long* __restrict__ total_out) {
    __shared__ unsigned s_wave[4];
    const long long n = n_dev ? *n_dev : n_imm;
    unsigned below = 0;
    for (int i = threadIdx.x; i < (int)blockIdx.x; i += 256) below += block_sums[i];
    unsigned add;
    (void)block_exclusive_scan_256(below, s_wave, add);  // (the total is what is wanted)
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0 && total_out)
        *total_out = (long long)add + (long long)block_sums[blockIdx.x];
    if (add == 0) return;
    const long long base = (long long)blockIdx.x * kScanChunk + (long long)threadIdx.x * 8;
#pragma unroll
    for (int i = 0; i < 8; ++i)
        if (base + i < n) vals[base + i] += add;
}

hipError_t launch_exclusive_scan(unsigned* vals, long long capacity, long long n_imm, const long long* n_dev,
                                 unsigned* block_sums, long long* total, hipStream_t s) {
    if (capacity <= kScanSmall) {
        hipLaunchKernelGGL(k_scan_small, dim3(1), dim3(256), 0, s, vals, n_imm, n_dev, total);
        return hipGetLastError();
    }
    long long blocks = (capacity + kScanChunk - 1) / kScanChunk;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(k_scan_local, dim3((unsigned)blocks), dim3(256), 0, s, vals, n_imm, n_dev, block_sums);
    if (blocks <= kScanTwoStep) {
        hipLaunchKernelGGL(k_scan_add_own, dim3((unsigned)blocks), dim3(256), 0, s, vals, n_imm, n_dev, block_sums,
                           total);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(k_scan_top, dim3(1), dim3(256), 0, s, block_sums, blocks, total);
    hipLaunchKernelGGL(k_scan_add, dim3((unsigned)blocks), dim3(256), 0, s, vals, n_imm, n_dev, block_sums);
    return hipGetLastError();
}

// ------------------------------------------------------------------ index build
// One thread per input row: set the row's bit; the first row of each word
// records its own index as that word's prefix.  Rows outside the grid are
// skipped and reported; a row not strictly above its predecessor is reported.
__global__ __launch_bounds__(256) void k_index_build(Geom g, const int32_t* __restrict__ coords, long long n_imm,
                                                     const long long* __restrict__ n_dev, long long n_cap,
                                                     unsigned long long* __restrict__ occ,
                                                     unsigned* __restrict__ occ_prefix, Counters* ctr) {
    long long n = n_dev ? *n_dev : n_imm;
    if (n > n_cap) n = n_cap;  // a device-resident count never reaches past the arrays
    if (n < 0) n = 0;
    const int stride = 1 + g.ndim;
    const int lane = threadIdx.x & 63;
    for (long long base = (long long)blockIdx.x * blockDim.x; base < n; base += (long long)gridDim.x * blockDim.x) {
        const long long r = base + threadIdx.x;
        long long key = -1;
        if (r < n) {
            int b, c0, c1, c2;
            load_site(g, coords + r * stride, b, c0, c1, c2);
            if (site_in_grid(g, b, c0, c1, c2)) {
                key = (long long)b * g.Npad + lin_of(g, c0, c1, c2);
                long long prev_key = -1;
                if (r > 0) {
                    int pb, p0, p1, p2;
                    load_site(g, coords + (r - 1) * stride, pb, p0, p1, p2);
                    if (site_in_grid(g, pb, p0, p1, p2)) prev_key = (long long)pb * g.Npad + lin_of(g, p0, p1, p2);
                }
                if (prev_key >= key) atomicOr(&ctr->flags, SCNN_FLAG_UNSORTED);
                if ((prev_key >> 6) != (key >> 6)) occ_prefix[key >> 6] = (unsigned)r;
            } else {
                atomicOr(&ctr->flags, SCNN_FLAG_BAD_COORD);
            }
        }
        // Sorted rows of one bitmap word sit in adjacent lanes: OR their bits together inside the wave and let the
        // first lane of each run issue the one atomic (a run may continue in the next wave, hence still atomic).
        const long long word = key >= 0 ? (key >> 6) : (long long)(-1 - lane);
        unsigned long long bits = key >= 0 ? (1ull << (key & 63)) : 0ull;
        const bool first = wave_or_runs(word, bits);
        if (key >= 0 && first) atomicOr(&occ[word], bits);
    }
}

hipError_t launch_index_build(const Geom& g, const int32_t* coords, long long n_imm, const long long* n_dev,
                              long long n_cap, unsigned long long* occ, unsigned* occ_prefix, Counters* ctr,
                              hipStream_t s) {
    long long blocks = (n_cap + 255) / 256;
    if (blocks < 1) blocks = 1;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(k_index_build, dim3((unsigned)blocks), dim3(256), 0, s, g, coords, n_imm, n_dev, n_cap, occ,
                       occ_prefix, ctr);
    return hipGetLastError();
}

// Everything that has to happen before the input is indexed, in one launch.  Block t < T prepares tap t of the
// filter: tap_active[t] = "has a non-zero weight", tap_coord[t] = its offset, and its weights in the layout of the
// convolution kernel that will run -- wb (matrix-core operand order:
// wb[((t * KC + kc) * NB + cb) * 64 + lane][s] = w[t][kc*32 + 8*gq + s][cb*16 + jj], lane = 16*gq + jj, so that a
// lane fetches its eight values of one (tap, kc, cb) with two 16-byte loads) or wp (fp64, rows padded to
// c_out_pad; the vector kernel).  The blocks from T on clear the zero-initialised part of the workspace.
// With `adjoint` set the filter is read as the one of the adjoint convolution (back-propagation to the data):
// `w` is then stored [T][c_out][c_in] and tap t of the adjoint is tap T-1-t of `w` (offset negated), i.e.
// element (t, ic, oc) = w[T-1-t][oc][ic].
__device__ inline float filter_at(const float* __restrict__ w, int T, int c_in, int c_out, int adjoint, int t, int ic,
                                  int oc) {
    return adjoint ? w[((size_t)(T - 1 - t) * c_out + oc) * c_in + ic] : w[((size_t)t * c_in + ic) * c_out + oc];
}

__global__ __launch_bounds__(256) void k_prepare(Geom g, const float* __restrict__ w, int c_in, int c_out, int adjoint,
                                                 int c_out_pad, double* __restrict__ wp, float* __restrict__ wb,
                                                 float* __restrict__ wq, int* __restrict__ tap_active,
                                                 int* __restrict__ tap_coord, uint4* __restrict__ zero_p,
                                                 size_t zero_n16) {
    if ((int)blockIdx.x >= g.T) {
        const size_t stride = (size_t)(gridDim.x - g.T) * blockDim.x;
        for (size_t i = (size_t)(blockIdx.x - g.T) * blockDim.x + threadIdx.x; i < zero_n16; i += stride)
            zero_p[i] = make_uint4(0, 0, 0, 0);
        return;
    }
    __shared__ int s_any;
    const int t = blockIdx.x;
    if (threadIdx.x == 0) s_any = 0;
    __syncthreads();
    int any = 0;
    if (wq) {
        // operand order of the quad kernel: [tap][32-channel chunk][channel / 4][lane][channel % 4], lane = output
        // channel (modulo 32 when there are at most 32 of them); channels and columns past the real ones are zero
        // With more than 64 output channels: one such filter per group of 64, one after the other.
        const int nch = (c_in + 31) / 32;
        const int n = nch * 2048;
        for (int col0 = 0; col0 < c_out; col0 += 64) {
            const int cg = c_out - col0 < 64 ? c_out - col0 : 64, cols = cg > 32 ? 64 : 32;
            float* wq_g = wq + (size_t)(col0 >> 6) * quad_filter_floats(g.T, c_in);
            for (int i = threadIdx.x; i < n; i += blockDim.x) {
                const int e = i & 3, lane = (i >> 2) & 63, j = (i >> 8) & 7, c = i >> 11;
                const int ic = c * 32 + 4 * j + e, oc = lane & (cols - 1);
                const float v =
                    (ic < c_in && oc < cg) ? filter_at(w, g.T, c_in, c_out, adjoint, t, ic, col0 + oc) : 0.0f;
                wq_g[(size_t)t * n + i] = v;
                any |= (v != 0.0f);
            }
        }
    } else if (wb) {
        // C_in = 16 is laid out like one 32-channel chunk: a lane's first four values are channels 4 gq .. 4 gq + 3,
        // its other four are zero
        const bool half = c_in == 16;
        const int nb = c_out / 16, n = (half ? 32 : c_in) * c_out;
        for (int i = threadIdx.x; i < n; i += blockDim.x) {
            const int sub = i & 7, lane = (i >> 3) & 63;
            const int r = i >> 9, cb = r % nb, kc = r / nb;  // (kc < C_in / 32 since n = (C_in / 32) * nb * 512)
            const int jj = lane & 15, gq = lane >> 4;
            const int ic = half ? (sub < 4 ? 4 * gq + sub : -1) : kc * 32 + 8 * gq + sub;
            const float v = ic >= 0 ? filter_at(w, g.T, c_in, c_out, adjoint, t, ic, cb * 16 + jj) : 0.0f;
            wb[(size_t)t * n + i] = v;
            any |= (v != 0.0f);
        }
    } else {
        const int n = c_in * c_out_pad;
        for (int i = threadIdx.x; i < n; i += blockDim.x) {
            const int ic = i / c_out_pad, oc = i % c_out_pad;
            float v = 0.0f;
            if (oc < c_out) v = filter_at(w, g.T, c_in, c_out, adjoint, t, ic, oc);
            wp[(size_t)t * n + i] = (double)v;
            any |= (v != 0.0f);
        }
    }
    if (any) s_any = 1;
    __syncthreads();
    if (threadIdx.x == 0) {
        tap_active[t] = s_any;
        // tap coordinates (t0, t1, t2), one byte each: delta = coordinate - H
        tap_coord[t] = (t / (g.K[2] * g.K[1])) | (((t / g.K[2]) % g.K[1]) << 8) | ((t % g.K[2]) << 16);
    }
}

hipError_t launch_prepare(const Geom& g, const float* w, int c_in, int c_out, int adjoint, int c_out_pad, double* wp,
                          float* wb, float* wq, int* tap_active, int* tap_coord, void* zero_p, size_t zero_bytes,
                          hipStream_t s) {
    const size_t n16 = (zero_bytes + 15) / 16;
    size_t zb = (n16 + 255) / 256;
    if (zb > 2048) zb = 2048;
    hipLaunchKernelGGL(k_prepare, dim3((unsigned)(g.T + zb)), dim3(256), 0, s, g, w, c_in, c_out, adjoint, c_out_pad, wp,
                       wb, wq, tap_active, tap_coord, (uint4*)zero_p, n16);
    return hipGetLastError();
}

// ------------------------------------------------------------------ candidate sites
// Candidate sites = occupied sites dilated by the filter's non-zero taps: an input at q reaches p = q - delta,
// i.e. p is a candidate iff some active tap has an occupied site at p + delta.  Sixteen lanes produce one 64-bit
// word of the candidate bitmap by OR-ing shifted windows of the occupancy bitmap (no atomics): each lane takes some
// of the (delta_0, delta_1) lines and the lanes combine with shuffles.  A word is cut
// into the runs it shares with grid lines (last axis); for a run and a (delta_0, delta_1) pair the source bits
// of all delta_2 lie in one window of at most three occupancy words.
__device__ inline unsigned long long funnel64(unsigned long long lo, unsigned long long hi, int s) {
    return s ? ((lo >> s) | (hi << (64 - s))) : lo;
}

// LANES lanes share one bitmap word, one (delta_0, delta_1) line at a time each: 16 on small grids, where one lane
// per word would leave most of the chip idle behind a chain of dependent loads, 1 on large grids.
template <int kDilateLanes>
__device__ __forceinline__ unsigned long long dilate_word(const Geom& g, const unsigned long long* __restrict__ occ,
                                                          const int* __restrict__ tap_active, long long w, int sub) {
    const int n_lines = g.K[0] * g.K[1];
    const int b = (int)(w / g.Wps);
    const long long p_first = (w - (long long)b * g.Wps) * 64;  // lin of bit 0
    long long remaining = g.N - p_first;                         // bits of this word that are sites
    if (remaining > 64) remaining = 64;
    unsigned long long out = 0;
    const long long sample_bit0 = (long long)b * g.Npad;
    const long long word_lo = (long long)b * g.Wps, word_hi = word_lo + g.Wps;  // this sample's words
    long long line = p_first / g.E[2];
    int c2 = (int)(p_first - line * g.E[2]);
    int c1 = (int)(line % g.E[1]), c0 = (int)(line / g.E[1]);
    int bit = 0;
    while (remaining > 0) {
        int len = g.E[2] - c2;
        if (len > remaining) len = (int)remaining;
        unsigned long long run = 0;
        for (int l = sub; l < n_lines; l += kDilateLanes) {
            const int t0 = l / g.K[1], t1 = l - t0 * g.K[1];
            const int q0 = c0 + t0 - g.H[0], q1 = c1 + t1 - g.H[1];
            if ((unsigned)q0 >= (unsigned)g.E[0] || (unsigned)q1 >= (unsigned)g.E[1]) continue;
            // window of occupancy bits [s - H2, s + len + H2) of line (q0, q1), s = site (q0, q1, c2)
            const long long s = sample_bit0 + ((long long)q0 * g.E[1] + q1) * g.E[2] + c2;
            const long long wb = (s - g.H[2]) >> 6;  // arithmetic shift: floor also for negatives
            unsigned long long win[3];
#pragma unroll
            for (int i = 0; i < 3; ++i) {
                const long long wi = wb + i;
                win[i] = (wi >= word_lo && wi < word_hi) ? occ[wi] : 0ull;
            }
            const int* act = tap_active + l * g.K[2];
            for (int t2 = 0; t2 < g.K[2]; ++t2) {
                if (!act[t2]) continue;
                const int d2 = t2 - g.H[2];
                // source z = c2 + i + d2 must stay on the line: i in [lo, hi)
                int lo = -d2 - c2, hi = g.E[2] - d2 - c2;
                if (lo < 0) lo = 0;
                if (hi > len) hi = len;
                if (lo >= hi) continue;
                const int o = (int)(s + d2 - wb * 64);  // 0 <= o < 128 for H2 <= 32
                unsigned long long bits = o < 64 ? funnel64(win[0], win[1], o) : funnel64(win[1], win[2], o - 64);
                unsigned long long m = (hi - lo) >= 64 ? ~0ull : (((1ull << (hi - lo)) - 1ull) << lo);
                run |= bits & m;
            }
        }
        out |= run << bit;
        bit += len;
        remaining -= len;
        c2 = 0;
        if (++c1 == g.E[1]) { c1 = 0; ++c0; }
    }
    // OR of the lanes' lines
    if constexpr (kDilateLanes > 1) {
#pragma unroll
        for (int d = 1; d < kDilateLanes; d <<= 1) out |= __shfl_xor(out, d, kDilateLanes);
    }
    return out;
}

template <int kDilateLanes>
__global__ __launch_bounds__(256) void k_cand_dilate(Geom g, const unsigned long long* __restrict__ occ,
                                                     const int* __restrict__ tap_active,
                                                     unsigned long long* __restrict__ cand,
                                                     unsigned* __restrict__ cand_count) {
    const long long n_words = (long long)g.batch * g.Wps;
    const int sub = threadIdx.x & (kDilateLanes - 1);
    const long long groups = (long long)gridDim.x * (blockDim.x / kDilateLanes);
    for (long long w = (long long)blockIdx.x * (blockDim.x / kDilateLanes) + threadIdx.x / kDilateLanes; w < n_words;
         w += groups) {
        const unsigned long long out = dilate_word<kDilateLanes>(g, occ, tap_active, w, sub);
        if (sub == 0) {
            cand[w] = out;
            cand_count[w] = (unsigned)__popcll(out);
        }
    }
}

// The same for bitmaps of up to kEmitMidWords words: a workgroup takes chunks of 256 / LANES consecutive words and also
// leaves each chunk's candidate count, from which k_cand_emit_mid finds its place in the candidate list without a
// scan launch in between.
template <int kDilateLanes>
__global__ __launch_bounds__(256) void k_cand_dilate_chunks(Geom g, const unsigned long long* __restrict__ occ,
                                                            const int* __restrict__ tap_active,
                                                            unsigned long long* __restrict__ cand,
                                                            unsigned* __restrict__ cand_count,
                                                            unsigned* __restrict__ chunk_sums) {
    constexpr int kChunk = 256 / kDilateLanes;
    __shared__ unsigned s_wave[4];
    const long long n_words = (long long)g.batch * g.Wps;
    const long long n_chunks = (n_words + kChunk - 1) / kChunk;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sub = threadIdx.x & (kDilateLanes - 1);
    for (long long c = blockIdx.x; c < n_chunks; c += gridDim.x) {
        const long long w = c * kChunk + threadIdx.x / kDilateLanes;
        unsigned n = 0;
        if (w < n_words) {
            const unsigned long long out = dilate_word<kDilateLanes>(g, occ, tap_active, w, sub);
            if (sub == 0) {
                n = (unsigned)__popcll(out);
                cand[w] = out;
                cand_count[w] = n;
            }
        }
#pragma unroll
        for (int d = 32; d > 0; d >>= 1) n += __shfl_xor(n, d, 64);
        if (lane == 0) s_wave[wave] = n;
        __syncthreads();
        if (threadIdx.x == 0) chunk_sums[c] = s_wave[0] + s_wave[1] + s_wave[2] + s_wave[3];
        __syncthreads();
    }
}

hipError_t launch_cand_dilate(const Geom& g, const unsigned long long* occ, const int* tap_active,
                              unsigned long long* cand, unsigned* cand_count, unsigned* chunk_sums, hipStream_t s) {
    const long long n_words = (long long)g.batch * g.Wps;
    const int lanes = cand_dilate_lanes(n_words, g.Wps);
    if (chunk_sums) {  // (the caller passes them for kEmitSmallWords < n_words <= kEmitMidWords)
        long long blocks = (n_words * lanes + 255) / 256;
        if (blocks > 8192) blocks = 8192;
        if (lanes == 16)
            hipLaunchKernelGGL(k_cand_dilate_chunks<16>, dim3((unsigned)blocks), dim3(256), 0, s, g, occ, tap_active,
                               cand, cand_count, chunk_sums);
        else
            hipLaunchKernelGGL(k_cand_dilate_chunks<1>, dim3((unsigned)blocks), dim3(256), 0, s, g, occ, tap_active,
                               cand, cand_count, chunk_sums);
        return hipGetLastError();
    }
    long long blocks = (n_words * lanes + 255) / 256;
    if (blocks < 1) blocks = 1;
    if (blocks > 8192) blocks = 8192;
    if (lanes == 16)
        hipLaunchKernelGGL(k_cand_dilate<16>, dim3((unsigned)blocks), dim3(256), 0, s, g, occ, tap_active, cand,
                           cand_count);
    else
        hipLaunchKernelGGL(k_cand_dilate<1>, dim3((unsigned)blocks), dim3(256), 0, s, g, occ, tap_active, cand,
                           cand_count);
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void k_popcount(const unsigned long long* __restrict__ bits, long long n_words,
                                                  unsigned* __restrict__ out) {
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n_words;
         i += (long long)gridDim.x * blockDim.x)
        out[i] = (unsigned)__popcll(bits[i]);
}

hipError_t launch_popcount(const unsigned long long* bits, long long n_words, unsigned* out, hipStream_t s) {
    long long blocks = (n_words + 255) / 256;
    if (blocks < 1) blocks = 1;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(k_popcount, dim3((unsigned)blocks), dim3(256), 0, s, bits, n_words, out);
    return hipGetLastError();
}

// Candidate list and its per-sample ranges, in one launch.
// Last block: per-sample candidate ranges and tile ranges.  Each sample's candidates are padded to whole tiles so
// that a tile never spans two samples.  rows16_start[b] = 16-row groups of all earlier samples (each sample
// rounded up), the unit in which the pair lists of the matrix-core path reserve their space.
// Other blocks, one thread per bitmap word: write the per-sample site index of every set bit at its rank.  The
// list comes out sorted by (b, lin).
__global__ __launch_bounds__(256) void k_cand_emit(Geom g, const unsigned long long* __restrict__ cand,
                                                   const unsigned* __restrict__ cand_prefix, long long n_words,
                                                   unsigned* __restrict__ cand_lin, long long cand_cap,
                                                   int* __restrict__ cand_start, int* __restrict__ tile_start,
                                                   int* __restrict__ rows16_start, Counters* ctr) {
    __shared__ unsigned s_wave[4];
    if (blockIdx.x == gridDim.x - 1) {
        const long long n_cand = ctr->n_cand;  // written by the scan
        const bool overflow = n_cand > cand_cap;
        for (int b = threadIdx.x; b <= g.batch; b += blockDim.x) {
            int v = 0;
            if (!overflow) v = (b == g.batch) ? (int)n_cand : (int)cand_prefix[(long long)b * g.Wps];
            cand_start[b] = v;
        }
        __syncthreads();
        const int n_tiles_all = sample_ranges_256(g.batch, cand_start, tile_start, rows16_start, s_wave);
        if (threadIdx.x == 0) {
            ctr->n_tiles = n_tiles_all;
            if (overflow) atomicOr(&ctr->flags, SCNN_FLAG_CAND_OVERFLOW);
        }
        return;
    }
    for (long long w = (long long)blockIdx.x * blockDim.x + threadIdx.x; w < n_words;
         w += (long long)(gridDim.x - 1) * blockDim.x) {
        unsigned long long bits = cand[w];
        if (!bits) continue;
        long long o = cand_prefix[w];
        const unsigned base = (unsigned)((w % g.Wps) * 64);
        while (bits) {
            const int bit = __ffsll((long long)bits) - 1;
            bits &= bits - 1;
            if (o < cand_cap) cand_lin[o] = base + (unsigned)bit;
            ++o;
        }
    }
}

// The same for short bitmaps (at most kEmitSmallWords words), without a scan launch before it: a block sums the counts
// of the words before its own (a few thousand numbers out of L2) and scans its 256 words itself; the last block scans
// the whole array once to find the per-sample ranges.  `cand_count` holds the words' candidate counts, unscanned.
__global__ __launch_bounds__(256) void k_cand_emit_small(Geom g, const unsigned long long* __restrict__ cand,
                                                         const unsigned* __restrict__ cand_count, int n_words,
                                                         unsigned* __restrict__ cand_lin, long long cand_cap,
                                                         int* __restrict__ cand_start, int* __restrict__ tile_start,
                                                         int* __restrict__ rows16_start, Counters* ctr) {
    __shared__ unsigned s_wave[4];
    if (blockIdx.x == gridDim.x - 1) {
        // exclusive scan in chunks of 2048 words; a sample starts at every Wps-th word
        unsigned carry = 0;
        for (int start = 0; start < n_words; start += kScanChunk) {
            const int base = start + threadIdx.x * 8;
            unsigned v[8], sum = 0;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                v[i] = (base + i < n_words) ? cand_count[base + i] : 0u;
                sum += v[i];
            }
            unsigned total;
            unsigned excl = carry + block_exclusive_scan_256(sum, s_wave, total);
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int w = base + i;
                if (w < n_words && w % (int)g.Wps == 0) cand_start[w / (int)g.Wps] = (int)excl;
                excl += v[i];
            }
            carry += total;
        }
        const long long n_cand = (long long)carry;
        const bool overflow = n_cand > cand_cap;
        __syncthreads();  // cand_start[0 .. batch) written
        if (overflow)
            for (int b = threadIdx.x; b < g.batch; b += blockDim.x) cand_start[b] = 0;
        if (threadIdx.x == 0) cand_start[g.batch] = overflow ? 0 : (int)n_cand;
        __syncthreads();
        const int n_tiles_all = sample_ranges_256(g.batch, cand_start, tile_start, rows16_start, s_wave);
        if (threadIdx.x == 0) {
            ctr->n_cand = n_cand;
            ctr->n_tiles = n_tiles_all;
            if (overflow) atomicOr(&ctr->flags, SCNN_FLAG_CAND_OVERFLOW);
        }
        return;
    }
    const int w0 = blockIdx.x * 256;
    unsigned below = 0;
    for (int i0 = threadIdx.x; i0 < w0; i0 += 256 * 8) {  // eight loads in flight per thread
        unsigned x[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) x[u] = i0 + 256 * u < w0 ? cand_count[i0 + 256 * u] : 0u;
#pragma unroll
        for (int u = 0; u < 8; ++u) below += x[u];
    }
    unsigned before_block;
    (void)block_exclusive_scan_256(below, s_wave, before_block);  // (the total is what is wanted)
    const int w = w0 + threadIdx.x;
    unsigned long long bits = w < n_words ? cand[w] : 0ull;
    unsigned block_total;
    long long o = (long long)before_block + block_exclusive_scan_256((unsigned)__popcll(bits), s_wave, block_total);
    const unsigned base = w < n_words ? (unsigned)((w % g.Wps) * 64) : 0u;
    while (bits) {
        const int bit = __ffsll((long long)bits) - 1;
        bits &= bits - 1;
        if (o < cand_cap) cand_lin[o] = base + (unsigned)bit;
        ++o;
    }
}

// The same for bitmaps of up to kEmitMidWords words, after k_cand_dilate_chunks: a block owns 256 words, adds up the
// counts of the chunks (of 1 << chunk_shift words: 256 or 16) before them, a few thousand numbers out of L2, and scans
// its own words.  The last
// block finds the per-sample ranges from the chunk counts by itself, so that no block waits for another.
// `cand_count` holds the words' candidate counts, unscanned.
__global__ __launch_bounds__(256) void k_cand_emit_mid(Geom g, const unsigned long long* __restrict__ cand,
                                                       const unsigned* __restrict__ cand_count,
                                                       const unsigned* __restrict__ chunk_sums, int chunk_shift,
                                                       long long n_words, unsigned* __restrict__ cand_lin,
                                                       long long cand_cap,
                                                       int* __restrict__ cand_start, int* __restrict__ tile_start,
                                                       int* __restrict__ rows16_start, Counters* ctr) {
    __shared__ unsigned s_wave[4];
    __shared__ unsigned long long s_total;
    __shared__ unsigned s_pref[kEmitMidChunks + 1];  // (last block) candidates in the chunks before chunk i
    if (blockIdx.x == gridDim.x - 1) {
        // exclusive scan of the chunk counts: a thread takes `per` consecutive chunks
        const int n_chunks = (int)((n_words + (1ll << chunk_shift) - 1) >> chunk_shift);  // (<= kEmitMidChunks)
        const int per = (n_chunks + 255) / 256, i_lo = (int)threadIdx.x * per;
        unsigned local = 0;
        for (int i = i_lo; i < i_lo + per && i < n_chunks; ++i) local += chunk_sums[i];
        unsigned total;
        unsigned run = block_exclusive_scan_256(local, s_wave, total);
        for (int i = i_lo; i < i_lo + per && i < n_chunks; ++i) {
            s_pref[i] = run;
            run += chunk_sums[i];
        }
        if (threadIdx.x == 0) {
            s_pref[n_chunks] = total;
            s_total = total;
        }
        __syncthreads();
        // candidates before sample b = chunks wholly before its first word + the words of the chunk it starts in
        for (int b = threadIdx.x; b <= g.batch; b += 256) {
            const long long w_b = (long long)b * g.Wps;  // (= n_words for b = batch)
            const int c_b = (int)(w_b >> chunk_shift);
            unsigned sum = s_pref[c_b];
            for (long long w0 = (long long)c_b << chunk_shift; w0 < w_b; w0 += 8) {  // eight loads in flight
                unsigned x[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) x[u] = w0 + u < w_b ? cand_count[w0 + u] : 0u;
#pragma unroll
                for (int u = 0; u < 8; ++u) sum += x[u];
            }
            // (a total beyond the capacity is far below 2^31: at most 2^31 sites per call)
            cand_start[b] = (int)sum;
        }
        __syncthreads();
        const long long n_cand = (long long)s_total;
        const bool overflow = n_cand > cand_cap;
        if (overflow)
            for (int b = threadIdx.x; b <= g.batch; b += blockDim.x) cand_start[b] = 0;
        __syncthreads();
        const int n_tiles_all = sample_ranges_256(g.batch, cand_start, tile_start, rows16_start, s_wave);
        if (threadIdx.x == 0) {
            ctr->n_cand = n_cand;
            ctr->n_tiles = n_tiles_all;
            if (overflow) atomicOr(&ctr->flags, SCNN_FLAG_CAND_OVERFLOW);
        }
        return;
    }
    const int c = blockIdx.x;  // words [256 c, 256 c + 256): whole chunks (a chunk has 256 or 16 words)
    const int chunks_below = (int)(((long long)c << 8) >> chunk_shift);
    unsigned below = 0;
    for (int i0 = threadIdx.x; i0 < chunks_below; i0 += 256 * 8) {  // eight loads in flight per thread
        unsigned x[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) x[u] = i0 + 256 * u < chunks_below ? chunk_sums[i0 + 256 * u] : 0u;
#pragma unroll
        for (int u = 0; u < 8; ++u) below += x[u];
    }
    unsigned before_block;
    (void)block_exclusive_scan_256(below, s_wave, before_block);  // (the total is what is wanted)
    const long long w = (long long)c * 256 + threadIdx.x;
    unsigned long long bits = w < n_words ? cand[w] : 0ull;
    unsigned block_total;
    long long o = (long long)before_block + block_exclusive_scan_256((unsigned)__popcll(bits), s_wave, block_total);
    const unsigned base = w < n_words ? (unsigned)((w % g.Wps) * 64) : 0u;
    while (bits) {
        const int bit = __ffsll((long long)bits) - 1;
        bits &= bits - 1;
        if (o < cand_cap) cand_lin[o] = base + (unsigned)bit;
        ++o;
    }
}

hipError_t launch_cand_emit_mid(const Geom& g, const unsigned long long* cand, const unsigned* cand_count,
                                const unsigned* chunk_sums, long long n_words, unsigned* cand_lin, long long cand_cap,
                                int* cand_start, int* tile_start, int* rows16_start, Counters* ctr, hipStream_t s) {
    const unsigned blocks = (unsigned)((n_words + 255) / 256);
    const int chunk_shift = cand_chunk_shift(n_words, g.Wps);
    hipLaunchKernelGGL(k_cand_emit_mid, dim3(blocks + 1), dim3(256), 0, s, g, cand, cand_count, chunk_sums,
                       chunk_shift, n_words, cand_lin, cand_cap, cand_start, tile_start, rows16_start, ctr);
    return hipGetLastError();
}

hipError_t launch_cand_emit(const Geom& g, const unsigned long long* cand, const unsigned* cand_prefix,
                            long long n_words, unsigned* cand_lin, long long cand_cap, int* cand_start,
                            int* tile_start, int* rows16_start, Counters* ctr, hipStream_t s) {
    long long blocks = (n_words + 255) / 256;
    if (blocks < 1) blocks = 1;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(k_cand_emit, dim3((unsigned)blocks + 1), dim3(256), 0, s, g, cand, cand_prefix, n_words,
                       cand_lin, cand_cap, cand_start, tile_start, rows16_start, ctr);
    return hipGetLastError();
}

hipError_t launch_cand_emit_small(const Geom& g, const unsigned long long* cand, const unsigned* cand_count,
                                  long long n_words, unsigned* cand_lin, long long cand_cap, int* cand_start,
                                  int* tile_start, int* rows16_start, Counters* ctr, hipStream_t s) {
    const unsigned blocks = (unsigned)((n_words + 255) / 256);
    hipLaunchKernelGGL(k_cand_emit_small, dim3(blocks + 1), dim3(256), 0, s, g, cand, cand_count, (int)n_words,
                       cand_lin, cand_cap, cand_start, tile_start, rows16_start, ctr);
    return hipGetLastError();
}

}  // namespace scnn
