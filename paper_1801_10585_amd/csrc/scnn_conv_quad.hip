// Matrix-core convolution, output-stationary over groups of four candidate sites (Alg. 1 steps 5-9, 13-14).
//
// A surface candidate has about a third of its taps' neighbours, and which ones differs from site to site.  The
// matrix instruction used here, v_mfma_f32_4x4x1_16b_f32 with its A operand broadcast to all blocks, multiplies FOUR
// rows by one input channel of a tap's weights for all output channels at once (lane = output channel): the unit
// that has to share a tap is a quad of sites instead of the sixteen rows of the larger instructions.  A wave owns 64
// consecutive candidate sites (half a response tile).  It looks up their neighbours, sorts the sites by their
// neighbour pattern so that a quad holds similar sites (a pattern-sorted quad has the neighbour in about 90 % of the
// (row, tap) slots it multiplies, against 45 % for sixteen consecutive rows), and then walks the taps: for every quad
// that has the tap it gathers the four neighbour rows (one buffer load; an absent neighbour is an out-of-range offset
// and reads as zero), runs one fp32 chain over at most 32 input channels, and adds the 4 x C_out results to fp64
// accumulators it keeps in registers for all its sites.  No partial sum ever leaves the wave: there are no atomics, the
// order of every addition is fixed by the data alone, and the result is reproducible bit for bit.  The fp32 matrix
// cores only ever add the at most 32 products of one (tap, 32-channel chunk); the long cancelling sum over taps and
// chunks is carried in double and rounded to fp32 once.
//
// Waves are independent (no workgroup barrier anywhere): a workgroup is just four of them sharing a launch slot.
#include <type_traits>

#include "scnn_internal.h"

namespace scnn {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

constexpr int kQuadWaves = 4;            // waves per workgroup
constexpr int kQuadRows = 64;            // candidate sites per wave
constexpr int kQuadMaxTaps = 32;         // taps per filter (one bit each in a site's neighbour pattern)
constexpr bool kQuadSingleChain = false;
constexpr int kQuadSteal = 2;            // XCDs after its own that a wave helps once its own has nothing left
constexpr int kQuadChunkMin = 128;       // shortest chunk (wave tiles)
constexpr int kQuadChunks = 8;           // chunks of wave tiles per XCD (see the kernel's tile order)
constexpr int kLineBatch = 9;            // filter lines whose bitmap words are fetched together
constexpr unsigned kAbsent = 0x80000000u;  // buffer offset of a neighbour that does not exist: out of range, reads 0

// LDS of one wave.  While the taps are walked: neighbour offsets [taps][64 sorted sites], the list of (tap, chunk)
// passes, the list of (pass, quad set) steps.  Afterwards the same bytes hold the 64 x C_out results for the
// transposition to the planar tile.
constexpr int kQuadTrWords = kQuadRows * 33;                              // transposition buffer: half the columns, padded rows
__host__ __device__ constexpr int quad_lds_words(int c_in, int taps) {
    const int nch = (c_in + 31) / 32;
    const int walk = taps * kQuadRows + taps * nch + (taps * nch * 16 + 4) + kQuadRows;
    return walk > kQuadTrWords ? walk : kQuadTrWords;
}
// Waves per SIMD the kernel is built for: its registers are the accumulators (64 sites x 64 channels, 4 or 8 bytes
// each) plus the weights of a pass.  Up to 32 input channels with fp32 sums fit 128 registers with ONE set of weights
// (reloaded between passes: the SIMD's other three waves cover the wait); the others hold two sets, one multiplying
// while the other is loaded.
__host__ __device__ constexpr int quad_waves_per_simd(int c_in, int qpm, int acc64) {
    if (c_in <= 32 && !acc64) return 4;
    return ((qpm == 1 && acc64) || c_in == 40 || c_in == 48) ? 2 : 3;  // (two chunk widths cost registers too)
}

// The fp32 products of one step: channel ch of the chunk is lane field kb = ch / NA of A register ch % NA (a lane
// loads NA consecutive channels), selected through the instruction's broadcast index.  Even and odd channels go to
// two accumulators, i.e. two independent chains of matrix instructions issued alternately: an instruction of a chain
// then never waits for the result of the one before it (its predecessor in the chain is two issue slots away).
template <int CH, int KC, int NA, int CBSZ>
__device__ __forceinline__ void quad_chain(const float (&a)[4], const float (&b)[32], f32x4& d0, f32x4& d1) {
    if constexpr (CH < KC) {
        if constexpr (CH % 2 == 0 || kQuadSingleChain)
            d0 = __builtin_amdgcn_mfma_f32_4x4x1f32(a[CH % NA], b[CH], d0, CBSZ, CH / NA, 0);
        else
            d1 = __builtin_amdgcn_mfma_f32_4x4x1f32(a[CH % NA], b[CH], d1, CBSZ, CH / NA, 0);
        quad_chain<CH + 1, KC, NA, CBSZ>(a, b, d0, d1);
    }
}

template <int NA>
__device__ __forceinline__ void quad_load_a(__amdgpu_buffer_rsrc_t rsrc, unsigned voff, unsigned soff, float (&a)[4]) {
    if constexpr (NA == 1) {
        a[0] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rsrc, voff, soff, 0));
    } else if constexpr (NA == 2) {
        const u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(rsrc, voff, soff, 0);
        a[0] = __uint_as_float(v.x);
        a[1] = __uint_as_float(v.y);
    } else {
        const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rsrc, voff, soff, 0);
        a[0] = __uint_as_float(v.x);
        a[1] = __uint_as_float(v.y);
        a[2] = __uint_as_float(v.z);
        a[3] = __uint_as_float(v.w);
    }
}

// Weights of one pass (tap, 32-channel chunk) in matrix-operand order: register ch of lane l holds
// w[tap][32 chunk + ch][column of lane l]; stored as [pass][ch / 4][lane][ch % 4] so that a wave reads 1 KiB runs.
template <int KC>
__device__ __forceinline__ void quad_load_b(const float* __restrict__ wq, int pass, int lane, float (&b)[32]) {
    const f32x4* p = (const f32x4*)(wq + (size_t)pass * 2048) + lane;
#pragma unroll
    for (int j = 0; j < (KC + 3) / 4; ++j) {
        const f32x4 v = p[j * 64];
        b[4 * j] = v.x;
        b[4 * j + 1] = v.y;
        b[4 * j + 2] = v.z;
        b[4 * j + 3] = v.w;
    }
}

// QPM = quads per matrix instruction: 1 (up to 64 output channels, lane = channel) or 2 (up to 32 output channels:
// the two half waves hold two quads that then have to share their taps).
// ACC64: the sums over taps and chunks are carried in fp64 (else fp32: for filters of few taps, where the additions
// across taps contribute less rounding error than the fp32 chains themselves).
template <int C_IN, int QPM, int ACC64>
__global__ __launch_bounds__(kQuadWaves * 64, quad_waves_per_simd(C_IN, QPM, ACC64)) void k_conv_quad(
    Geom g, const unsigned long long* __restrict__ occ, const unsigned* __restrict__ occ_prefix, long long nnz_in,
    const float* __restrict__ feats, const float* __restrict__ wq, const float* __restrict__ bias, int c_out,
    int col0, int c_out_all, const int* __restrict__ tap_active, const unsigned* __restrict__ cand_lin,
    const int* __restrict__ cand_start, const int* __restrict__ tile_start, Counters* __restrict__ ctr,
    float* __restrict__ resp) {
    // c_out: the output channels of this launch (at most 64), col0 .. col0 + c_out - 1 of the layer's c_out_all; wq
    // and bias point at this group's; the group col0 / 64 has its own tile counters
    constexpr int NCH = (C_IN + 31) / 32;        // 32-channel chunks
    constexpr int KB = 16 / QPM;                 // lanes of a quad row that hold channels
    constexpr int NS = 16 / QPM;                 // quad sets (4 * QPM sites that share their taps) per wave
    constexpr int SET = 4 * QPM;                 // sites per quad set
    constexpr int CBSZ = QPM == 1 ? 4 : 3;       // A broadcast over 16 or 8 blocks
    constexpr int COLS = 64 / QPM;
    constexpr int KC_LAST = C_IN - 32 * (NCH - 1);
    // channels a lane loads per row: those of a full chunk and of the last chunk (three become four: 16-byte loads)
    constexpr int NA_FULL = 32 / KB, NA_LAST = (KC_LAST + KB - 1) / KB == 3 ? 4 : (KC_LAST + KB - 1) / KB;
    constexpr int NA0 = NCH == 1 ? NA_LAST : NA_FULL;  // of every chunk but the last (of the only chunk)
    static_assert(NA_FULL <= 4 && NA_LAST <= 4 && NA_LAST >= 1, "chunk width");
    const int LDSW = quad_lds_words(C_IN, g.T);
    typedef typename std::conditional<ACC64 != 0, double, float>::type acc_t;
    extern __shared__ __align__(16) unsigned smem_u[];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    unsigned* s_tab = smem_u + wave * LDSW;                    // [taps][64] buffer offsets, sorted site order
    unsigned* s_pass = s_tab + g.T * kQuadRows;                  // [passes] tap | chunk << 8 | mask of quad sets << 16
    unsigned* s_step = s_pass + g.T * NCH;            // [steps + 2] (tap * 64 + set * SET) * 4 | chunk << 20
    unsigned* s_pos = s_step + (g.T * NCH * 16 + 4);  // [64] sorted position of a site
    float* s_tr = (float*)s_tab;                               // [64][COLS / 2 + 1] after the walk
    const unsigned long long lt_mask = (1ull << lane) - 1ull;

    // lane fields of the matrix operands
    const int row_in_set = (lane & 3) + 4 * (QPM == 2 ? (lane >> 5) : 0);
    const int kb = (lane >> 2) & (KB - 1);
    const __amdgpu_buffer_rsrc_t rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void*)feats, 0, (int)(nnz_in * (long long)(C_IN * 4)), 0x00020000);

    // taps with a non-zero weight, one bit each
    const unsigned act_mask = (unsigned)__ballot(lane < g.T && tap_active[lane < g.T ? lane : 0] != 0);

    // XCD-aware order: workgroup i runs on XCD i % kXcds.  The wave tiles are cut into kXcds * kQuadChunks chunks of
    // equal length and XCD x owns the chunks x, x + kXcds, x + 2 kXcds, ...: inside a chunk neighbouring tiles share input rows,
    // which then stay in that XCD's L2, and because an XCD's chunks are spread over the whole batch, samples whose
    // sites cost more (more taps per quad) are shared out evenly instead of falling to two or three XCDs.  An XCD's
    // wave tiles are numbered through its chunks (v = 0, 1, ...).
    //
    // Units of work.  A wave tile keeps a wave busy for as long as a third of a small layer's whole launch, so what
    // is left for a last, partial round of the XCD's wave slots would leave most of the chip waiting for a few
    // waves.  The wave tiles of that round are therefore dealt out in halves or quarters (32 or 16 of the 64 sites:
    // the other sites are treated like sites past the sample's end, and the unit stores only its own) when that
    // still gives every piece a slot of its own.  A site's sum does not depend on the sites it shares a quad with
    // (an absent neighbour adds an exact zero), so the split does not change a single bit of the result.
    // A wave starts with unit u = its slot and then draws further units from its XCD's counter, and from the next
    // XCDs' once its own is used up.
    const int n_wt = 2 * (int)ctr->n_tiles;
    const int xcd = blockIdx.x % kXcds, slot = (blockIdx.x / kXcds) * kQuadWaves + wave, per_xcd = (gridDim.x / kXcds) * kQuadWaves;
    // (only where every chunk gets at least kQuadChunkMin wave tiles: shorter chunks lose more at their ends,
    // where the neighbours' rows belong to another XCD's L2, than the even shares win - measured on 16 -> 32
    // channels over 3900 wave tiles: 113 us in one chunk per XCD, 117 us in three)
    const int n_chunks = n_wt >= kXcds * kQuadChunks * kQuadChunkMin ? kQuadChunks : 1;
    const int chunk = n_wt > 0 ? (n_wt + kXcds * n_chunks - 1) / (kXcds * n_chunks) : 1;
    // unit u of XCD x: its wave tile (-1 past the end: then every later unit of that XCD is past the end as well) and
    // the sites lo .. hi - 1 of it
    auto unit_of = [&](int x, int u, int& lo, int& hi) {
        int vspan = 0;  // wave tiles of XCD x
        for (int c = 0; c < n_chunks; ++c) {
            const int left = n_wt - (c * kXcds + x) * chunk;
            vspan += left <= 0 ? 0 : (left < chunk ? left : chunk);
        }
        lo = 0;
        hi = kQuadRows;
        const int whole = (vspan / per_xcd) * per_xcd, rest = vspan - whole;
        const int sl = rest * 4 <= per_xcd ? 2 : (rest * 2 <= per_xcd ? 1 : 0);
        int v = u;
        if (u >= whole) {
            const int r = u - whole;
            v = whole + (r >> sl);
            lo = (r & ((1 << sl) - 1)) * (kQuadRows >> sl);
            hi = lo + (kQuadRows >> sl);
        }
        if (v >= vspan) return -1;
        const int c = v / chunk;
        return (c * kXcds + x) * chunk + (v - c * chunk);
    };
    unsigned* tickets = ctr->conv_ticket + (col0 >> 6) * kXcds * kTicketStride;

    int row_lo = 0, row_hi = kQuadRows, lo_next = 0, hi_next = 0;
    bool own_done = unit_of(xcd, per_xcd, lo_next, hi_next) < 0;  // nothing to draw beyond the first units
    for (int wt = unit_of(xcd, slot, row_lo, row_hi); wt >= 0;) {
        const int tile = wt >> 1, half = wt & 1;
        const int b = sample_of_tile(tile_start, g.batch, tile);
        const int first = cand_start[b] + (tile - tile_start[b]) * kTileRows + half * kQuadRows;
        int nrows = cand_start[b + 1] - first;
        nrows = nrows > kQuadRows ? kQuadRows : nrows;

        acc_t acc[NS][4];
#pragma unroll
        for (int s = 0; s < NS; ++s)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[s][r] = (acc_t)0;
        unsigned my_pos = (unsigned)lane;  // sorted position of site `lane` (of the wave's 64)

        if (nrows > row_lo) {
            // ---- neighbours of site `lane`: buffer offsets into s_tab[tap][lane], pattern bits into `mask`.
            //      The taps of one filter line (t0, t1, .) look at adjacent sites, which sit in at most two adjacent
            //      words of the occupancy bitmap: both words and their row prefixes are fetched for kLineBatch lines
            //      at a time, all loads in flight together, and the lines' taps are resolved from them afterwards.
            int c0 = 0, c1 = 0, c2 = 0;
            const bool live = lane < nrows && lane >= row_lo && lane < row_hi;
            if (live) site_of(g, cand_lin[first + lane], c0, c1, c2);
            unsigned mask = 0;
            // LDS address of s_tab[0][lane], made opaque per tile: the addresses of the table's rows must not be
            // computed once for the whole kernel and kept in registers
            unsigned tab_w = (unsigned)(size_t)s_tab + (unsigned)lane * 4u;
            asm volatile("" : "+v"(tab_w));
            const int n_lines = g.K[0] * g.K[1];
            const unsigned w_last = (unsigned)g.batch * (unsigned)g.Wps - 1u;
            const int q2s = c2 - g.H[2];                       // site of tap k of a line is q2s + k
            const int k_lo = q2s < 0 ? -q2s : 0;               // first tap whose site is on the line
            for (int line0 = 0; line0 < n_lines; line0 += kLineBatch) {
                unsigned long long word_a[kLineBatch], word_b[kLineBatch];
                unsigned pre_a[kLineBatch], pre_b[kLineBatch], bit0[kLineBatch], w_rel[kLineBatch];
                bool ok[kLineBatch];
#pragma unroll
                for (int i = 0; i < kLineBatch; ++i) {
                    const int line = line0 + i < n_lines ? line0 + i : n_lines - 1;
                    const int t0 = line / g.K[1], t1 = line - t0 * g.K[1];
                    const int q0 = c0 + t0 - g.H[0], q1 = c1 + t1 - g.H[1];
                    ok[i] = live && line0 + i < n_lines && (unsigned)q0 < (unsigned)g.E[0] && (unsigned)q1 < (unsigned)g.E[1];
                    bit0[i] = (unsigned)((q0 * g.E[1] + q1) * g.E[2]);  // site index of (q0, q1, 0), if ok
                    const unsigned first_bit = ok[i] ? bit0[i] + (unsigned)(q2s + k_lo) : 0u;
                    w_rel[i] = first_bit >> 6;
                    const unsigned w0 = (unsigned)b * (unsigned)g.Wps + w_rel[i];
                    const unsigned wa = ok[i] ? (w0 < w_last ? w0 : w_last) : 0u, wb = wa < w_last ? wa + 1u : wa;
                    word_a[i] = occ[wa];
                    word_b[i] = occ[wb];
                    pre_a[i] = occ_prefix[wa];
                    pre_b[i] = occ_prefix[wb];
                }
                // A line's taps sit next to each other in the bitmap: bit k of `win` = site of tap k occupied, valid
                // (on the line, tap active).  The row of a present tap = rows before the window + present taps below it.
#pragma unroll
                for (int i = 0; i < kLineBatch; ++i) {
                    if (line0 + i >= n_lines) break;
                    const int tap0 = (line0 + i) * g.K[2];
                    const unsigned first_bit = bit0[i] + (unsigned)(q2s + k_lo);
                    const unsigned p = first_bit & 63u;   // position of the window's first site in word_a
                    unsigned long long both = word_a[i] >> p;
                    if (p) both |= word_b[i] << (64u - p);
                    // taps on the line: k_lo <= k < min(K2, E2 - q2s); and active
                    const int k_hi = g.E[2] - q2s < g.K[2] ? g.E[2] - q2s : g.K[2];
                    unsigned valid = (k_hi >= 32 ? ~0u : ((1u << (k_hi > 0 ? k_hi : 0)) - 1u)) & ~((1u << k_lo) - 1u);
                    valid &= act_mask >> tap0;
                    const unsigned raw = (unsigned)both << k_lo;      // occupancy of the sites the taps look at
                    const unsigned win = ok[i] ? raw & valid : 0u;    // ... where the tap counts
                    mask |= win << tap0;
                    // rows before the window in word_a; taps from bit s_k on lie in word_b, whose own prefix counts
                    // from its first bit (every occupied site is a row, whether or not its tap counts)
                    const unsigned s_k = 64u - p + (unsigned)k_lo;
                    const unsigned base_a = pre_a[i] + (unsigned)__popcll(word_a[i] & ((1ull << p) - 1ull));
                    const unsigned base_b = pre_b[i] - (unsigned)__popc(s_k >= 32u ? raw : raw & ((1u << s_k) - 1u));
                    for (int k = 0; k < g.K[2]; ++k) {
                        const unsigned row = ((unsigned)k < s_k ? base_a : base_b) + (unsigned)__popc(raw & ((1u << k) - 1u));
                        const unsigned off = ((win >> k) & 1u) ? row * (unsigned)(C_IN * 4) : kAbsent;
                        *(__attribute__((address_space(3))) unsigned*)(size_t)(tab_w + (unsigned)(tap0 + k) * 256u) = off;
                    }
                }
            }
            // ---- sort the sites by pattern (bitonic network over the wave; ties by site, so the order is a
            //      function of the data alone)
            unsigned key = mask, orig_s = (unsigned)lane;  // orig_s: the site that sits at sorted position `lane`
#pragma unroll
            for (int k = 2; k <= 64; k <<= 1)
#pragma unroll
                for (int j = k >> 1; j > 0; j >>= 1) {
                    const unsigned ok = __shfl_xor(key, j, 64), oo = __shfl_xor(orig_s, j, 64);
                    const bool other_less = ok < key || (ok == key && oo < orig_s);
                    const bool want_min = ((lane & k) == 0) == ((lane & j) == 0);
                    if (other_less == want_min) {
                        key = ok;
                        orig_s = oo;
                    }
                }
            s_pos[orig_s] = (unsigned)lane;
            my_pos = s_pos[lane];
            // rows of the table into sorted order, in place (a wave's LDS reads finish before its next writes)
            for (int t = 0; t < g.T; ++t) {
                const unsigned v = s_tab[t * 64 + lane];
                s_tab[t * 64 + my_pos] = v;
            }
            // ---- taps of each quad set = union over its sites; step list: per tap, per chunk, the sets that have it
            unsigned u = key;
            u |= __shfl_xor(u, 1, 64);
            u |= __shfl_xor(u, 2, 64);
            if constexpr (QPM == 2) u |= __shfl_xor(u, 4, 64);
            const bool leader = (lane & (SET - 1)) == 0;
            int n_pass = 0, n_step = 0;
            for (int t = 0; t < g.T; ++t) {
                const unsigned long long m = __ballot(leader && ((u >> t) & 1u));
                if (m == 0ull) continue;
                const int cnt = __popcll(m);
                // bit s of the pass entry = quad set s has the tap (the leaders sit SET lanes apart)
                // the leaders' bits, SET lanes apart, moved next to each other: bit st = set st has the tap
                unsigned long long x = m;
                if constexpr (QPM == 1) {
                    x = (x | x >> 3) & 0x0303030303030303ull;
                    x = (x | x >> 6) & 0x000f000f000f000full;
                    x = (x | x >> 12) & 0x000000ff000000ffull;
                    x = (x | x >> 24) & 0xffffull;
                } else {
                    x = (x | x >> 7) & 0x0003000300030003ull;
                    x = (x | x >> 14) & 0x0000000f0000000full;
                    x = (x | x >> 28) & 0xffull;
                }
                const unsigned set_bits = (unsigned)x;
#pragma unroll
                for (int c = 0; c < NCH; ++c) {
                    if (lane == 0) s_pass[n_pass + c] = (unsigned)t | (unsigned)c << 8 | set_bits << 16;
                    if (leader && ((u >> t) & 1u))
                        s_step[n_step + c * cnt + __popcll(m & lt_mask)] =
                            (unsigned)((t * 64 + lane) * 4) | (unsigned)c << 20;
                }
                n_pass += NCH;
                n_step += NCH * cnt;
            }
            if (lane < 3) s_step[n_step + lane] = 0u;  // read ahead by the pipeline, never multiplied

            if (n_step > 0) {
                // ---- the walk.  Pipeline per step: list entry two steps ahead (LDS), the set's neighbour offsets one
                //      step ahead (LDS), the gathered rows one step ahead (buffer load).
                float a_next[4], b0[32], b1[32];
                const unsigned tab_lane = (unsigned)(size_t)s_tab + (unsigned)row_in_set * 4u;  // LDS byte address
                const unsigned kb_off = (unsigned)kb * 4u;  // times NA below: a lane loads NA consecutive channels
                auto tab_at = [&](unsigned e) {
                    return *(const __attribute__((address_space(3))) unsigned*)(size_t)(tab_lane + (e & 0xffffu));
                };
                // (the chunk's byte offset goes into the checked vector offset: an offset past the array reads as 0)
                auto load_a = [&](unsigned off, unsigned e, float (&a)[4]) {
                    const unsigned chunk = (e >> 20) & 3u;
                    if (NCH > 1 && NA_LAST != NA0 && chunk == NCH - 1)
                        quad_load_a<NA_LAST>(rsrc, off + (kb_off * NA_LAST + chunk * 128u), 0u, a);
                    else
                        quad_load_a<NA0>(rsrc, off + (kb_off * NA0 + chunk * 128u), 0u, a);
                };
                // at the top of step n: a_next = rows of step n, (e_1, off_1) = list entry and neighbour offsets of step
                // n + 1, e_raw = list entry of step n + 2 as it comes from LDS (made uniform a step after it was read)
                const unsigned e_first = __builtin_amdgcn_readfirstlane(s_step[0]);
                unsigned e_1 = __builtin_amdgcn_readfirstlane(s_step[1]);
                load_a(tab_at(e_first), e_first, a_next);
                unsigned off_1 = tab_at(e_1);
                unsigned e_raw = s_step[2];
                int step = 0;
                // One step = one quad set against one pass: the chain, then the set's four (per lane) fp64 additions.
                // The sets are walked by straight-line code, one copy per set, so that the accumulators are plain
                // registers; which sets a pass has comes from its mask.
                auto run_step = [&](const float (&bw)[32], acc_t (&ac)[4], bool last_chunk) {
                    float a_cur[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) a_cur[i] = a_next[i];
                    // rows of the next step; offsets of the one after; list entry of the one after that
                    load_a(off_1, e_1, a_next);
                    e_1 = __builtin_amdgcn_readfirstlane(e_raw);
                    off_1 = tab_at(e_1);
                    e_raw = s_step[step + 3];
                    ++step;
                    f32x4 d0 = {0.f, 0.f, 0.f, 0.f}, d1 = {0.f, 0.f, 0.f, 0.f};
                    if (NCH == 1 || last_chunk)
                        quad_chain<0, KC_LAST, NA_LAST, CBSZ>(a_cur, bw, d0, d1);
                    else
                        quad_chain<0, 32, NA_FULL, CBSZ>(a_cur, bw, d0, d1);
#pragma unroll
                    for (int r = 0; r < 4; ++r) ac[r] += (acc_t)(d0[r] + d1[r]);
                };
                auto run_pass = [&](const float (&bw)[32], unsigned pass_info) {
                    const unsigned sets = pass_info >> 16;
                    const bool last_chunk = NCH > 1 && ((pass_info >> 8) & 0xffu) == NCH - 1;
#pragma unroll
                    for (int st = 0; st < NS; ++st)
                        if (sets & (1u << st)) run_step(bw, acc[st], last_chunk);
                };
                auto pass_index = [&](unsigned info) { return (int)(info & 0xffu) * NCH + (int)((info >> 8) & 0xffu); };
                auto load_pass = [&](unsigned info, float (&bw)[32]) {
                    if (NCH > 1 && ((info >> 8) & 0xffu) != NCH - 1)
                        quad_load_b<32>(wq, pass_index(info), lane, bw);
                    else
                        quad_load_b<KC_LAST>(wq, pass_index(info), lane, bw);
                };
                if constexpr (quad_waves_per_simd(C_IN, QPM, ACC64) >= 4) {
                    // one register set: the next pass's weights are asked for when the last step of this pass has
                    // been issued; the SIMD's other waves cover the wait
                    unsigned p_info = __builtin_amdgcn_readfirstlane(s_pass[0]);
                    load_pass(p_info, b0);
                    for (int p = 0; p < n_pass; ++p) {
                        run_pass(b0, p_info);
                        if (p + 1 < n_pass) {
                            p_info = __builtin_amdgcn_readfirstlane(s_pass[p + 1]);
                            load_pass(p_info, b0);
                        }
                    }
                } else {
                // passes in pairs: one register set multiplies while the other receives the next pass's weights
                unsigned p_info = __builtin_amdgcn_readfirstlane(s_pass[0]);
                load_pass(p_info, b0);
                for (int p = 0; p < n_pass; p += 2) {
                    unsigned p_next = 0;
                    if (p + 1 < n_pass) {
                        p_next = __builtin_amdgcn_readfirstlane(s_pass[p + 1]);
                        load_pass(p_next, b1);
                    }
                    run_pass(b0, p_info);
                    if (p + 1 >= n_pass) break;
                    if (p + 2 < n_pass) {
                        p_info = __builtin_amdgcn_readfirstlane(s_pass[p + 2]);
                        load_pass(p_info, b0);
                    }
                    run_pass(b1, p_next);
                }
                }
            }
        }

        // ---- next tile: ask the own span's counter now and look at the answer after the epilogue, which hides the
        //      round trip.  (Lane 0 asks; the counters sit on separate cache lines.)
        unsigned ticket = 0;
        if (!own_done && lane == 0) ticket = atomicAdd(&tickets[xcd * kTicketStride], 1u);

        // ---- epilogue: one rounding to fp32, bias on the non-zero entries, transposition through LDS to the planar
        //      tile: a lane holds its channel's values of all sorted positions and writes them in that order (fixed
        //      offsets); then lane = site reads the row of its sorted position.  Sites past the sample's end store 0.
        //      The buffer holds half of the columns at a time.
        {
            constexpr int HC = COLS / 2;                         // columns per half
            const int col = lane & (COLS - 1), colh = col & (HC - 1);
            const float bv = (bias && col < c_out) ? bias[col] : 0.0f;
            float* tr_w = s_tr + colh + (QPM == 2 ? 4 * (HC + 1) * (lane >> 5) : 0);
            const float* tr_r = s_tr + my_pos * (HC + 1);
            float* dst = resp + ((size_t)tile * c_out_all + col0) * kTileRows + half * kQuadRows + lane;
            const bool mine = lane >= row_lo && lane < row_hi;  // (the unit's own sites)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                if ((col >= HC) == (h == 1)) {
                    if (bias) {
#pragma unroll
                        for (int st = 0; st < NS; ++st)
#pragma unroll
                            for (int r = 0; r < 4; ++r) {
                                float x = (float)acc[st][r];
                                if (x != 0.0f) x += bv;
                                tr_w[(st * SET + r) * (HC + 1)] = x;
                            }
                    } else {
#pragma unroll
                        for (int st = 0; st < NS; ++st)
#pragma unroll
                            for (int r = 0; r < 4; ++r) tr_w[(st * SET + r) * (HC + 1)] = (float)acc[st][r];
                    }
                }
                const int c_end = c_out < (h + 1) * HC ? c_out : (h + 1) * HC;
                int c = h * HC;
                for (; c + 8 <= c_end; c += 8) {
                    float v[8];
#pragma unroll
                    for (int i = 0; i < 8; ++i) v[i] = tr_r[c - h * HC + i];
                    if (mine) {
#pragma unroll
                        for (int i = 0; i < 8; ++i) dst[(size_t)(c + i) * kTileRows] = v[i];
                    }
                }
                for (; c < c_end; ++c) {
                    const float v = tr_r[c - h * HC];
                    if (mine) dst[(size_t)c * kTileRows] = v;
                }
            }
        }
        int next_wt = -1;
        if (!own_done) {
            next_wt = unit_of(xcd, per_xcd + (int)__builtin_amdgcn_readfirstlane(ticket), lo_next, hi_next);
            own_done = next_wt < 0;
        }
        if (own_done) {
            // the own units are used up: help the next XCDs, so that none ends long before the others (tiles differ
            // in work).  Only the next two are tried: a wave that finds nothing there retires.
            int got = -1;
            if (lane == 0) {
                for (int d = 1; d <= kQuadSteal && got < 0; ++d) {
                    const int x = (xcd + d) % kXcds;
                    if (unit_of(x, per_xcd, lo_next, hi_next) < 0) continue;  // (an XCD with nothing to draw)
                    got = unit_of(x, per_xcd + (int)atomicAdd(&tickets[x * kTicketStride], 1u), lo_next, hi_next);
                }
            }
            next_wt = __builtin_amdgcn_readfirstlane(got);
            lo_next = __builtin_amdgcn_readfirstlane(lo_next);
            hi_next = __builtin_amdgcn_readfirstlane(hi_next);
        }
        row_lo = lo_next;
        row_hi = hi_next;
        wt = next_wt;
    }
}

bool conv_quad_supported(const Geom& g, int c_in, int c_out, long long nnz_in) {
    if (g.T > kQuadMaxTaps) return false;
    const bool shape = (c_in == 8 || c_in == 16 || c_in == 24 || c_in == 32 || c_in == 40 || c_in == 48 || c_in == 64 ||
                        c_in == 96 || c_in == 128) &&
                       c_out >= 1 && c_out <= kQuadMaxCout;
    return shape && nnz_in > 0 && nnz_in * (long long)c_in * 4 < (1ll << 31);
}

template <int C_IN, int QPM, int ACC64>
static hipError_t launch_conv_quad_t(const Geom& g, const unsigned long long* occ, const unsigned* occ_prefix,
                                     long long nnz_in, const float* feats, const float* wq, const float* bias, int c_out,
                                     int col0, int c_out_all, const int* tap_active, const unsigned* cand_lin,
                                     const int* cand_start, const int* tile_start, Counters* ctr, float* resp, int cus,
                                     hipStream_t s) {
    const size_t lds = (size_t)quad_lds_words(C_IN, g.T) * 4 * kQuadWaves;
    hipError_t e = hipFuncSetAttribute((const void*)k_conv_quad<C_IN, QPM, ACC64>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    // one workgroup (four waves) per SIMD wave slot of every CU, as far as the CU's 160 KiB of LDS hold them (every
    // workgroup must be resident: they are persistent); a multiple of kXcds: one span of tiles per XCD
    int per_cu = quad_waves_per_simd(C_IN, QPM, ACC64);
    if ((size_t)per_cu * lds > 160 * 1024) per_cu = (int)((160 * 1024) / lds);
    const int grid = (cus * per_cu + kXcds - 1) / kXcds * kXcds;
    hipLaunchKernelGGL((k_conv_quad<C_IN, QPM, ACC64>), dim3(grid), dim3(kQuadWaves * 64), lds, s, g, occ, occ_prefix,
                       nnz_in, feats, wq, bias, c_out, col0, c_out_all, tap_active, cand_lin, cand_start, tile_start, ctr,
                       resp);
    return hipGetLastError();
}

hipError_t launch_conv_quad(const Geom& g, const unsigned long long* occ, const unsigned* occ_prefix, long long nnz_in,
                            const float* feats, int c_in, const float* wq, int c_out, const float* bias,
                            const int* tap_active, const unsigned* cand_lin, const int* cand_start,
                            const int* tile_start, Counters* ctr, float* resp, int cus, hipStream_t s) {
    // fp32 sums over taps for filters of at most 32 (tap, chunk) passes (a 3x3x3 filter over up to 32 channels),
    // fp64 sums beyond
    const bool acc64 = (long long)g.T * ((c_in + 31) / 32) > 32;
    // more than 64 output channels: one launch per group of 64 (a wave's accumulators hold 64 sites x 64 channels);
    // every group repeats the look-ups and the sort, which the wider layers' matrix work outweighs
    for (int col0 = 0; col0 < c_out; col0 += 64) {
        const int cg = c_out - col0 < 64 ? c_out - col0 : 64;
        const float* wq_g = wq + (size_t)(col0 >> 6) * quad_filter_floats(g.T, c_in);
        const float* bias_g = bias ? bias + col0 : nullptr;
        hipError_t e = hipErrorInvalidValue;
#define SCNN_QUAD_ARGS g, occ, occ_prefix, nnz_in, feats, wq_g, bias_g, cg, col0, c_out, tap_active, cand_lin, cand_start, tile_start, ctr, resp, cus, s
#define SCNN_QUAD_CASE(CI)                                                                                            \
    if (c_in == CI) {                                                                                                 \
        if (cg > 32)                                                                                                  \
            e = acc64 ? launch_conv_quad_t<CI, 1, 1>(SCNN_QUAD_ARGS) : launch_conv_quad_t<CI, 1, 0>(SCNN_QUAD_ARGS);  \
        else                                                                                                          \
            e = acc64 ? launch_conv_quad_t<CI, 2, 1>(SCNN_QUAD_ARGS) : launch_conv_quad_t<CI, 2, 0>(SCNN_QUAD_ARGS);  \
    }
        SCNN_QUAD_CASE(8) SCNN_QUAD_CASE(16) SCNN_QUAD_CASE(24) SCNN_QUAD_CASE(32) SCNN_QUAD_CASE(40) SCNN_QUAD_CASE(48)
        SCNN_QUAD_CASE(64) SCNN_QUAD_CASE(96) SCNN_QUAD_CASE(128)
#undef SCNN_QUAD_CASE
#undef SCNN_QUAD_ARGS
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace scnn
