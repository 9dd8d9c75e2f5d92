// Host side of the C ABI: argument checks, workspace layout, launch sequences.
// Nothing here touches values; every step of the layer runs in the kernels.
#include <atomic>
#include <cmath>
#include <cstddef>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <vector>

#include "scnn_internal.h"

namespace scnn {

static thread_local char g_err[256] = "";
// Kernel family of the convolution step, per calling thread:
// 0 = by shape and size, 1 = always the vector kernels, 2 = matrix cores wherever a matrix-core kernel takes the shape,
// 3 = the pair-list matrix-core kernel where it takes the shape (else the vector kernels).
static thread_local int g_conv_path = 0;
static thread_local const char* g_last_conv_kernel = "";

enum class ConvKernel { kValu, kPair, kQuad };

// Which kernel multiplies.  The quad kernel (output-stationary, registers only) takes C_in in {8, .., 64} and up to
// 128 output channels (a launch per 64) with at most 32 taps, also C_in = 96 and 128 where the pair-list kernel does
// not take the output width; the pair-list kernel remains for more than 32 taps and for 96 and 128 input channels.  With 8, 16 or 24 input channels the matrix cores pay only on layers of enough tiles (128 or 1024, by
// shape) with enough output channels; narrower and smaller layers are faster on the vector kernels.
static ConvKernel conv_kernel_for(const Geom& g, int c_in, int c_out, long long nnz_in, long long tiles_cap) {
    if (g_conv_path == 1) return ConvKernel::kValu;
    const bool pair_ok = conv_mfma_supported(g, c_in, c_out, nnz_in);
    if (g_conv_path == 3) return pair_ok ? ConvKernel::kPair : ConvKernel::kValu;
    const bool quad_ok = conv_quad_supported(g, c_in, c_out, nnz_in);
    if (g_conv_path == 2) return quad_ok ? ConvKernel::kQuad : (pair_ok ? ConvKernel::kPair : ConvKernel::kValu);
    // 8, 16 and 24 input channels pay for the matrix-core kernels' look-ups and lists only on layers whose rows carry
    // enough multiply-adds per neighbour: C_in x C_out of at least 256 with at least 24 output channels (8->32,
    // 16->24), or of at least 384 (24->16); narrower layers (8->8, 8->16, 16->16: the first blocks of the paper's
    // networks) are faster on the vector kernels.  The layer must also be large enough: 128 tiles for 16 or 24 input
    // and at least 24 output channels (four samples of 16^3 with every site a candidate: 16->24 35 -> 31 us, 24->24
    // 43 -> 33 us; at 64 tiles the vector kernels' 32-row form wins, 24 against 32 us), 1024 tiles for the others
    const int mac = c_in * c_out;
    const long long min_tiles = (c_in >= 16 && c_out >= 24) ? 128 : 1024;
    const bool wide = c_in >= 32 || ((c_in == 8 || c_in == 16 || c_in == 24) && tiles_cap >= min_tiles &&
                                     ((mac >= 256 && c_out >= 24) || mac >= 384));
    // 96 and 128 input channels: three or four chunks per tap put the quad kernel's sums in fp64 registers (two waves
    // per SIMD); where the pair-list kernel takes the shape it is 10-35 % faster there, and the quad kernel takes
    // what it does not (output channels beyond 64 or no multiple of 16), which used to fall to the vector kernels
    if (pair_ok && wide && c_in > 64) return ConvKernel::kPair;
    if (quad_ok && wide) return ConvKernel::kQuad;
    if (pair_ok && wide) return ConvKernel::kPair;
    return ConvKernel::kValu;
}

static int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

static int fail_hip(hipError_t e, const char* what) {
    return fail(SCNN_EHIP, "%s: %s", what, hipGetErrorString(e));
}

#define SCNN_TRY(expr)                                         \
    do {                                                       \
        hipError_t e__ = (expr);                               \
        if (e__ != hipSuccess) return fail_hip(e__, #expr);    \
    } while (0)

static constexpr long long kMaxIndex = 0x7fffffffLL;  // rows, candidates and sites use 31-bit indices
static constexpr int kMaxChannels = 1024;

// Right-align the real axes in three internal axes.
static int make_geom(int ndim, const int32_t* extent, int batch, const int32_t* ksize, Geom* g) {
    if (ndim != 2 && ndim != 3) return fail(SCNN_EINVAL, "ndim must be 2 or 3 (got %d)", ndim);
    if (!extent) return fail(SCNN_EINVAL, "extent is null");
    if (batch < 1) return fail(SCNN_EINVAL, "batch must be >= 1 (got %d)", batch);
    memset(g, 0, sizeof(*g));
    g->ndim = ndim;
    g->batch = batch;
    for (int a = 0; a < 3; ++a) { g->E[a] = 1; g->K[a] = 1; g->H[a] = 0; }
    long long n = 1;
    for (int a = 0; a < ndim; ++a) {
        if (extent[a] < 1) return fail(SCNN_EINVAL, "extent[%d] = %d", a, extent[a]);
        g->E[3 - ndim + a] = extent[a];
        n *= extent[a];
        if (n > kMaxIndex) return fail(SCNN_ECAPACITY, "more than 2^31-1 sites per sample");
    }
    long long t = 1;
    if (ksize) {
        for (int a = 0; a < ndim; ++a) {
            if (ksize[a] < 1 || ksize[a] % 2 == 0) return fail(SCNN_EINVAL, "ksize[%d] = %d must be odd", a, ksize[a]);
            if (ksize[a] > 63) return fail(SCNN_ECAPACITY, "ksize[%d] = %d exceeds 63", a, ksize[a]);
            g->K[3 - ndim + a] = ksize[a];
            g->H[3 - ndim + a] = (ksize[a] - 1) / 2;
            t *= ksize[a];
            if (t > 1 << 20) return fail(SCNN_ECAPACITY, "filter has too many taps");
        }
    }
    g->T = (int)t;
    g->N = n;
    g->Npad = round_up(n, 64);
    g->Wps = (int)(g->Npad / 64);
    if ((long long)batch * g->Wps > kMaxIndex) return fail(SCNN_ECAPACITY, "batch * sites too large");
    return SCNN_OK;
}

static Geom pooled_geom(const Geom& g) {
    Geom p = g;
    long long n = 1;
    for (int a = 0; a < 3; ++a) {
        p.E[a] = (g.E[a] + 1) / 2;
        p.K[a] = 1;
        p.H[a] = 0;
        n *= p.E[a];
    }
    p.T = 1;
    p.N = n;
    p.Npad = round_up(n, 64);
    p.Wps = (int)(p.Npad / 64);
    return p;
}

// Bump allocator over the caller's workspace; with base == nullptr it only measures.
struct Carver {
    char* base;
    size_t off = 0;
    explicit Carver(void* b) : base((char*)b) {}
    template <typename T>
    T* take(size_t count) {
        off = (off + 255) & ~(size_t)255;
        T* p = base ? (T*)(base + off) : nullptr;
        off += count * sizeof(T);
        return p;
    }
    size_t total() const { return (off + 255) & ~(size_t)255; }
};

static long long scan_blocks(long long cap) { return (cap + kScanChunk - 1) / kScanChunk + 2; }

static long long default_cand_bound(const Geom& g, long long nnz_in) {
    const long long grid = (long long)g.batch * g.N;
    const long long reach = nnz_in * (long long)g.T;
    return grid < reach ? grid : reach;
}


// ---------------------------------------------------------------- per-stage timing (measurement support)
// Stages 0..6 belong to sparse_conv_fwd, stages 7..11 to sparse_conv_bwd.
static const char* const kStageNames[] = {"index_build", "candidates", "conv_prepare", "conv", "topk_select",
                                          "compact_write", "pool_finish", "bwd_index", "bwd_pairs", "bwd_data_conv",
                                          "bwd_data_write", "bwd_filter"};
static constexpr int kFwdStages = 7, kBwdStages = 5, kStages = kFwdStages + kBwdStages;
struct ProfCall {
    hipEvent_t ev[kFwdStages + 1];
    int first_stage, n_stages;
    unsigned recorded;  // bit i: ev[i] was recorded in this call
};
static constexpr int kConvStage = 3;  // "conv": the only stage timed in mode 2
static thread_local int g_prof_on = 0;  // 0 off, 1 every stage boundary, 2 only the convolution stage's two,
                                        // 3 the same on every fourth forward call
static thread_local unsigned g_prof_tick = 0;
static thread_local std::vector<ProfCall>* g_prof_calls = nullptr;   // recorded, not yet collected
static thread_local std::vector<ProfCall>* g_prof_pool = nullptr;    // idle events for reuse

struct StageTimer {
    ProfCall call;
    bool on = false, only_conv = false;
    int next = 0;
    hipStream_t s;
    StageTimer(hipStream_t stream, int first_stage, int n_stages) : s(stream) {
        if (!g_prof_on) return;
        if (g_prof_on == 3 && (first_stage != 0 || (g_prof_tick++ & 3u) != 0)) return;
        if (!g_prof_calls) g_prof_calls = new std::vector<ProfCall>();
        if (!g_prof_pool) g_prof_pool = new std::vector<ProfCall>();
        if (!g_prof_pool->empty()) {
            call = g_prof_pool->back();
            g_prof_pool->pop_back();
        } else {
            for (int i = 0; i <= kFwdStages; ++i)
                if (hipEventCreate(&call.ev[i]) != hipSuccess) return;
        }
        call.first_stage = first_stage;
        call.n_stages = n_stages;
        call.recorded = 0;
        only_conv = g_prof_on >= 2 && first_stage == 0;
        on = true;
    }
    void mark() {  // boundary between stage next-1 and stage next
        if (on && next <= call.n_stages) {
            if (!only_conv || next == kConvStage || next == kConvStage + 1) {
                (void)hipEventRecord(call.ev[next], s);
                call.recorded |= 1u << next;
            }
            ++next;
        }
    }
    void done() {
        if (!on) return;
        while (next <= call.n_stages) mark();
        g_prof_calls->push_back(call);
        on = false;
    }
};

// ---------------------------------------------------------------- sparse_conv_fwd
struct ConvWs {
    // zeroed at the start of every call (contiguous)
    Counters* ctr;
    unsigned long long* occ;
    unsigned long long* cand;
    unsigned long long* pbits;
    unsigned long long* occ_sel;
    ColState* cols;
    unsigned long long* tile_state;
    size_t zero_bytes;
    // not zeroed
    uint2* part;
    unsigned long long* row_keep;
    unsigned long long* row_plane;
    long long* tile_base;
    unsigned* occ_prefix;
    unsigned* cand_prefix;
    unsigned* pprefix;
    unsigned* block_sums;
    int* cand_start;
    int* tile_start;
    int* rows16_start;
    int* tap_active;
    int* tap_coord;
    double* wp;
    unsigned* cand_lin;
    float* resp;
    uint2* side;
    unsigned long long side_cap;
    unsigned* pairs;
    unsigned short* block_tap;
    float* wb;
    float* wq;
    uint2* tile_hdr;
    long long block_cap;
    ConvKernel kernel;
    int32_t* tmp_coords;
    float* tmp_feats;
    long long* pool_key;
    size_t total;
    long long cand_cap, tiles_cap, pool_cap;
    int c_out_pad;
};

static void carve_conv(void* base, const Geom& g, const Geom& gp, long long nnz_in, int c_in, int c_out, unsigned fuse,
                       long long cand_cap, ConvWs* w) {
    Carver c(base);
    const long long nw = (long long)g.batch * g.Wps;
    const long long nwp = (long long)gp.batch * gp.Wps;
    const bool pool = (fuse & SCNN_FUSE_MAXPOOL2) != 0;
    const long long ncols = (long long)g.batch * c_out;
    w->cand_cap = cand_cap;
    w->tiles_cap = (cand_cap + kTileRows - 1) / kTileRows + g.batch;
    const long long grid_p = (long long)gp.batch * gp.N;
    w->pool_cap = cand_cap < grid_p ? cand_cap : grid_p;
    w->c_out_pad = (int)round_up(c_out, 16);
    w->ctr = c.take<Counters>(1);
    w->occ = c.take<unsigned long long>(nw);
    w->cand = c.take<unsigned long long>(nw);
    w->pbits = c.take<unsigned long long>(pool ? nwp : 0);
    w->occ_sel = c.take<unsigned long long>(pool ? nw : 0);  // occupancy of the selected rows, for the pooling
    // rows known to survive are marked during the selection when the streaming compaction kernel can use them
    const bool marks = !topk_small_columns(g) && c_out > kMarkMinChannels && c_out <= kMarkPlanes;
    w->cols = c.take<ColState>(ncols);
    w->tile_state = c.take<unsigned long long>(w->tiles_cap);
    w->zero_bytes = c.total();
    w->part = c.take<uint2>(topk_small_columns(g) ? 0 : ncols * kTopkPartWords);
    w->row_keep = c.take<unsigned long long>(marks ? 2 * w->tiles_cap : 0);
    w->row_plane = c.take<unsigned long long>(marks ? 2 * w->tiles_cap * kMarkPlanes : 0);
    w->tile_base = c.take<long long>(marks ? w->tiles_cap : 0);
    w->occ_prefix = c.take<unsigned>(nw);
    w->cand_prefix = c.take<unsigned>(nw);
    w->pprefix = c.take<unsigned>(pool ? nwp : 0);
    long long sb = scan_blocks(nw);
    if (nw <= kEmitMidWords && cand_chunk_count(nw, g.Wps) > sb) sb = cand_chunk_count(nw, g.Wps);  // per-chunk candidate counts
    if (scan_blocks(w->tiles_cap) > sb) sb = scan_blocks(w->tiles_cap);
    if (scan_blocks(nwp) > sb) sb = scan_blocks(nwp);
    if (nwp <= kEmitMidWords && (nwp + 255) / 256 > sb) sb = (nwp + 255) / 256;  // (the pooling's chunk counts)
    w->block_sums = c.take<unsigned>(sb);
    w->cand_start = c.take<int>(g.batch + 1);
    w->tile_start = c.take<int>(g.batch + 1);
    w->rows16_start = c.take<int>(g.batch + 1);
    w->tap_active = c.take<int>(g.T);
    w->tap_coord = c.take<int>(g.T);
    w->wp = c.take<double>((size_t)g.T * c_in * w->c_out_pad);
    w->cand_lin = c.take<unsigned>(cand_cap);
    w->resp = c.take<float>((size_t)w->tiles_cap * c_out * kTileRows);
    w->side_cap = (unsigned long long)w->tiles_cap * kTileRows * c_out;
    w->side = c.take<uint2>((size_t)w->side_cap);
    w->kernel = conv_kernel_for(g, c_in, c_out, nnz_in, w->tiles_cap);
    // pair-list kernel: every (input row, tap) gives at most one pair; a tile reserves whole blocks per active tap
    w->block_cap = w->kernel == ConvKernel::kPair ? (long long)g.T * (cand_cap / 16 + w->tiles_cap) : 0;
    w->pairs = c.take<unsigned>((size_t)w->block_cap * 16);
    w->block_tap = c.take<unsigned short>((size_t)w->block_cap);
    w->wb = c.take<float>(w->block_cap ? (size_t)g.T * round_up(c_in, 32) * c_out : 0);
    w->tile_hdr = c.take<uint2>(w->block_cap ? w->tiles_cap : 0);
    w->wq = c.take<float>(w->kernel == ConvKernel::kQuad ? quad_groups(c_out) * quad_filter_floats(g.T, c_in) : 0);
    w->tmp_coords = c.take<int32_t>(pool ? (size_t)cand_cap * (1 + g.ndim) : 0);
    w->tmp_feats = c.take<float>(pool ? (size_t)cand_cap * c_out : 0);
    w->pool_key = c.take<long long>(pool ? w->pool_cap : 0);
    w->total = c.total();
    (void)nnz_in;
}

static int check_conv_sizes(const Geom& g, long long nnz_in, int c_in, int c_out, long long* cand_cap) {
    if (nnz_in < 0 || nnz_in > kMaxIndex) return fail(SCNN_ECAPACITY, "nnz_in = %lld out of range", nnz_in);
    if (c_in < 1 || c_out < 1) return fail(SCNN_EINVAL, "channel counts must be positive");
    if (c_in > kMaxChannels || c_out > kMaxChannels) return fail(SCNN_ECAPACITY, "at most %d channels", kMaxChannels);
    long long bound = default_cand_bound(g, nnz_in);
    if (*cand_cap <= 0 || *cand_cap > bound) *cand_cap = bound;
    if (*cand_cap < 1) *cand_cap = 1;
    if (*cand_cap + (long long)g.batch * kTileRows > kMaxIndex) return fail(SCNN_ECAPACITY, "too many candidate sites");
    return SCNN_OK;
}

}  // namespace scnn

using namespace scnn;

extern "C" {

const char* scnn_last_error(void) { return g_err; }
int scnn_version(void) { return 1; }

int64_t scnn_k_from_rho(double rho_up, int64_t n_sites) {
    if (!(rho_up >= 0.0) || n_sites < 0) return 0;
    const double x = rho_up * (double)n_sites;
    const double rx = std::floor(x + 0.5);
    int64_t k = (std::fabs(x - rx) <= 1e-9 * (x > 1.0 ? x : 1.0)) ? (int64_t)rx : (int64_t)std::floor(x);
    if (k < 0) k = 0;
    if (k > n_sites) k = n_sites;
    return k;
}

int64_t sparse_conv_fwd_max_rows(int ndim, const int32_t* extent, int batch, int64_t nnz_in, const int32_t* ksize) {
    Geom g;
    int rc = make_geom(ndim, extent, batch, ksize, &g);
    if (rc != SCNN_OK) return rc;
    if (!ksize) return fail(SCNN_EINVAL, "ksize is null");
    if (nnz_in < 0) return fail(SCNN_EINVAL, "nnz_in < 0");
    return default_cand_bound(g, nnz_in);
}

size_t sparse_conv_fwd_workspace(int ndim, const int32_t* extent, int batch, int64_t nnz_in, int c_in, int c_out,
                                 const int32_t* ksize, unsigned fuse, int64_t cand_capacity) {
    Geom g;
    if (!ksize || make_geom(ndim, extent, batch, ksize, &g) != SCNN_OK) return 0;
    long long cap = cand_capacity;
    if (check_conv_sizes(g, nnz_in, c_in, c_out, &cap) != SCNN_OK) return 0;
    ConvWs w;
    carve_conv(nullptr, g, pooled_geom(g), nnz_in, c_in, c_out, fuse, cap, &w);
    return w.total;
}

static int conv_fwd_impl(int ndim, const int32_t* extent, int batch, const int32_t* in_coords, const float* in_feats,
                         int64_t nnz_in, const int64_t* nnz_in_dev, int c_in, const int32_t* ksize, const float* w,
                         const float* bias, int c_out, double rho_up, int topk_mode, unsigned fuse,
                         int32_t* out_coords, float* out_feats, int64_t out_capacity, int64_t cand_capacity,
                         int64_t* nnz_out, void* workspace, size_t workspace_bytes, void* hip_stream) {
    Geom g;
    if (!ksize) return fail(SCNN_EINVAL, "ksize is null");
    int rc = make_geom(ndim, extent, batch, ksize, &g);
    if (rc != SCNN_OK) return rc;
    long long cap = cand_capacity;
    rc = check_conv_sizes(g, nnz_in, c_in, c_out, &cap);
    if (rc != SCNN_OK) return rc;
    if (!(rho_up >= 0.0 && rho_up <= 1.0)) return fail(SCNN_EINVAL, "rho_up = %g not in [0, 1]", rho_up);
    if (topk_mode != SCNN_TOPK_ABS && topk_mode != SCNN_TOPK_SIGNED) return fail(SCNN_EINVAL, "bad topk_mode");
    if (fuse & ~(SCNN_FUSE_RELU | SCNN_FUSE_MAXPOOL2)) return fail(SCNN_EINVAL, "unknown fuse bits");
    if (!w || !nnz_out || !workspace) return fail(SCNN_EINVAL, "null pointer (w, nnz_out or workspace)");
    if (nnz_in > 0 && (!in_coords || !in_feats)) return fail(SCNN_EINVAL, "null input arrays");
    if (out_capacity < 0 || out_capacity > kMaxIndex) return fail(SCNN_EINVAL, "bad out_capacity");
    if (out_capacity > 0 && (!out_coords || !out_feats)) return fail(SCNN_EINVAL, "null output arrays");
    if (((uintptr_t)workspace & 255) != 0) return fail(SCNN_EWORKSPACE, "workspace must be 256-byte aligned");
    const Geom gp = pooled_geom(g);
    ConvWs ws;
    carve_conv(workspace, g, gp, nnz_in, c_in, c_out, fuse, cap, &ws);
    if (ws.total > workspace_bytes)
        return fail(SCNN_EWORKSPACE, "workspace too small: %zu < %zu bytes", workspace_bytes, ws.total);
    hipStream_t s = (hipStream_t)hip_stream;
    const long long k = scnn_k_from_rho(rho_up, g.N);
    const long long nw = (long long)g.batch * g.Wps;
    const bool pool = (fuse & SCNN_FUSE_MAXPOOL2) != 0;
    const int relu = (fuse & SCNN_FUSE_RELU) ? 1 : 0;

    StageTimer timer(s, 0, kFwdStages);
    timer.mark();
    // the matrix-core kernels load input rows 16 bytes at a time
    const ConvKernel kernel = ((uintptr_t)in_feats & 15) == 0 ? ws.kernel : ConvKernel::kValu;
    SCNN_TRY(launch_prepare(g, w, c_in, c_out, 0, ws.c_out_pad, ws.wp, kernel == ConvKernel::kPair ? ws.wb : nullptr,
                            kernel == ConvKernel::kQuad ? ws.wq : nullptr, ws.tap_active, ws.tap_coord, workspace,
                            ws.zero_bytes, s));
    // with a device-resident count, nnz_in is only the capacity of the input arrays: rows past the true count are
    // never indexed, so no look-up can return them
    SCNN_TRY(launch_index_build(g, in_coords, nnz_in, (const long long*)nnz_in_dev, nnz_in, ws.occ, ws.occ_prefix,
                                ws.ctr, s));
    timer.mark();
    const bool emit_mid = nw > kEmitSmallWords && nw <= kEmitMidWords;
    SCNN_TRY(launch_cand_dilate(g, ws.occ, ws.tap_active, ws.cand, ws.cand_prefix, emit_mid ? ws.block_sums : nullptr, s));
    if (nw <= kEmitSmallWords) {
        SCNN_TRY(launch_cand_emit_small(g, ws.cand, ws.cand_prefix, nw, ws.cand_lin, ws.cand_cap, ws.cand_start,
                                        ws.tile_start, ws.rows16_start, ws.ctr, s));
    } else if (emit_mid) {
        SCNN_TRY(launch_cand_emit_mid(g, ws.cand, ws.cand_prefix, ws.block_sums, nw, ws.cand_lin, ws.cand_cap,
                                      ws.cand_start, ws.tile_start, ws.rows16_start, ws.ctr, s));
    } else {
        SCNN_TRY(launch_exclusive_scan(ws.cand_prefix, nw, nw, nullptr, ws.block_sums, &ws.ctr->n_cand, s));
        SCNN_TRY(launch_cand_emit(g, ws.cand, ws.cand_prefix, nw, ws.cand_lin, ws.cand_cap, ws.cand_start,
                                  ws.tile_start, ws.rows16_start, ws.ctr, s));
    }
    timer.mark();
    if (kernel == ConvKernel::kQuad) {
        const int cus = device_cu_count();
        timer.mark();
        SCNN_TRY(launch_conv_quad(g, ws.occ, ws.occ_prefix, nnz_in, in_feats, c_in, ws.wq, c_out, bias, ws.tap_active,
                                  ws.cand_lin, ws.cand_start, ws.tile_start, ws.ctr, ws.resp, cus, s));
        g_last_conv_kernel = "k_conv_quad";
    } else if (kernel == ConvKernel::kPair) {
        SCNN_TRY(launch_pair_build(g, ws.occ, ws.occ_prefix, nnz_in, ws.tap_active, ws.tap_coord, ws.cand_lin,
                                   ws.cand_start, ws.tile_start, ws.rows16_start, ws.ctr, ws.pairs, ws.block_tap,
                                   ws.tile_hdr, ws.block_cap, ws.tiles_cap, nullptr, s));
        timer.mark();
        SCNN_TRY(launch_conv_mfma(g, nnz_in, in_feats, c_in, ws.wb, c_out, bias, ws.pairs, ws.block_tap, ws.tile_hdr,
                                  ws.ctr, ws.resp, s));
        g_last_conv_kernel = "k_conv_mfma";
    } else {
        timer.mark();
        SCNN_TRY(launch_conv_valu(g, ws.occ, ws.occ_prefix, nnz_in, in_feats, c_in, ws.wp, c_out, ws.c_out_pad, bias,
                                  ws.tap_active, ws.cand_lin, ws.cand_start, ws.tile_start, ws.ctr, ws.tiles_cap,
                                  ws.resp, s));
        g_last_conv_kernel = "k_conv_valu";
    }
    timer.mark();
    const bool marks = !topk_small_columns(g) && c_out > kMarkMinChannels && c_out <= kMarkPlanes && k > 0;
    SCNN_TRY(launch_topk(g, c_out, k, topk_mode, relu, ws.tile_start, ws.resp, ws.cols, ws.side, ws.part,
                         marks ? ws.row_keep : nullptr, marks ? ws.row_plane : nullptr, marks ? ws.tile_base : nullptr,
                         ws.tiles_cap, ws.ctr, s));
    timer.mark();
    if (!pool) {
        SCNN_TRY(launch_select_write(g, c_out, topk_mode, relu, ws.cand_start, ws.tile_start, ws.cand_lin, ws.resp,
                                     ws.cols, ws.tile_state, ws.tiles_cap, ws.ctr, out_coords, out_feats,
                                     out_capacity, (long long*)nnz_out, 0, 1, marks ? ws.tile_base : nullptr, s));
        timer.mark();
    } else {
        SCNN_TRY(launch_select_write(g, c_out, topk_mode, relu, ws.cand_start, ws.tile_start, ws.cand_lin, ws.resp,
                                     ws.cols, ws.tile_state, ws.tiles_cap, ws.ctr, ws.tmp_coords, ws.tmp_feats,
                                     ws.cand_cap, nullptr, 0, 0, marks ? ws.tile_base : nullptr, s));
        timer.mark();
        SCNN_TRY(launch_maxpool(g, gp, ws.tmp_coords, ws.tmp_feats, 0, &ws.ctr->n_rows, ws.cand_cap, c_out, 1,
                                ws.occ_sel, ws.occ_prefix, ws.pbits, ws.pprefix, ws.block_sums, ws.pool_key,
                                ws.pool_cap, out_coords, out_feats, out_capacity, ws.ctr, (long long*)nnz_out, 0, 1,
                                s));
    }
    timer.done();
    return SCNN_OK;
}

// ---------------------------------------------------------------- sparse_conv_bwd
namespace {
struct BwdWs {
    Counters* ctr;
    unsigned long long* occ;  // occupancy of the gradient rows
    size_t zero_bytes;
    unsigned* occ_prefix;
    int* cand_start;
    int* tile_start;
    int* rows16_start;
    int* tap_active;
    int* tap_coord;
    double* wp;
    unsigned* cand_lin;
    float* resp;
    unsigned* pairs;
    unsigned short* block_tap;
    float* wb;
    uint2* tile_hdr;
    unsigned short* tap_first;
    double* fpart;
    long long block_cap, tiles_cap;
    int c_in_pad, chunks_mfma, chunks_valu;
    bool mfma_shape;
    size_t total;
};
void carve_bwd(void* base, const Geom& g, long long nnz_in, int c_in, int c_out, long long g_rows, BwdWs* w) {
    Carver c(base);
    const long long nw = (long long)g.batch * g.Wps;
    const long long n_elem = (long long)g.T * c_in * c_out;
    w->tiles_cap = (nnz_in + kTileRows - 1) / kTileRows + g.batch;
    w->c_in_pad = (int)round_up(c_in, 16);
    // the adjoint convolution contracts over C_out and produces C_in channels
    w->mfma_shape = conv_mfma_supported(g, c_out, c_in, g_rows) && bwd_filter_mfma_supported(c_in, c_out, g_rows);
    w->chunks_mfma = w->mfma_shape ? bwd_filter_chunks(g, c_in, c_out, w->tiles_cap, true) : 0;
    w->chunks_valu = bwd_filter_chunks(g, c_in, c_out, w->tiles_cap, false);
    w->ctr = c.take<Counters>(1);
    w->occ = c.take<unsigned long long>(nw);
    w->zero_bytes = c.total();
    w->occ_prefix = c.take<unsigned>(nw);
    w->cand_start = c.take<int>(g.batch + 1);
    w->tile_start = c.take<int>(g.batch + 1);
    w->rows16_start = c.take<int>(g.batch + 1);
    w->tap_active = c.take<int>(g.T);
    w->tap_coord = c.take<int>(g.T);
    w->wp = c.take<double>((size_t)g.T * c_out * w->c_in_pad);
    w->cand_lin = c.take<unsigned>(nnz_in > 0 ? nnz_in : 1);
    w->resp = c.take<float>((size_t)w->tiles_cap * c_in * kTileRows);
    w->block_cap = w->mfma_shape ? (long long)g.T * (nnz_in / 16 + w->tiles_cap) : 0;
    w->pairs = c.take<unsigned>((size_t)w->block_cap * 16);
    w->block_tap = c.take<unsigned short>((size_t)w->block_cap);
    // (the adjoint filter in matrix-operand order: its input channels, C_out, padded to a whole 32-channel chunk)
    w->wb = c.take<float>(w->mfma_shape ? (size_t)g.T * round_up(c_out, 32) * c_in : 0);
    w->tile_hdr = c.take<uint2>(w->mfma_shape ? w->tiles_cap : 0);
    w->tap_first = c.take<unsigned short>(w->mfma_shape ? (size_t)w->tiles_cap * (g.T + 1) : 0);
    const int chunks = w->chunks_mfma > w->chunks_valu ? w->chunks_mfma : w->chunks_valu;
    w->fpart = c.take<double>((size_t)chunks * n_elem);
    w->total = c.total();
}
int check_bwd_sizes(const Geom& g, long long nnz_in, int c_in, int c_out, long long g_rows) {
    if (nnz_in < 0 || nnz_in > kMaxIndex - (long long)g.batch * kTileRows)
        return fail(SCNN_ECAPACITY, "nnz_in = %lld out of range", nnz_in);
    if (g_rows < 0 || g_rows > kMaxIndex) return fail(SCNN_ECAPACITY, "g_rows = %lld out of range", g_rows);
    if (c_in < 1 || c_out < 1) return fail(SCNN_EINVAL, "channel counts must be positive");
    if (c_in > kMaxChannels || c_out > kMaxChannels) return fail(SCNN_ECAPACITY, "at most %d channels", kMaxChannels);
    if ((long long)g.T * c_in * c_out > kMaxIndex) return fail(SCNN_ECAPACITY, "filter too large");
    return SCNN_OK;
}
}  // namespace

size_t sparse_conv_bwd_workspace(int ndim, const int32_t* extent, int batch, int64_t nnz_in, int c_in, int c_out,
                                 const int32_t* ksize, int64_t g_rows) {
    Geom g;
    if (!ksize || make_geom(ndim, extent, batch, ksize, &g) != SCNN_OK) return 0;
    if (check_bwd_sizes(g, nnz_in, c_in, c_out, g_rows) != SCNN_OK) return 0;
    BwdWs w;
    carve_bwd(nullptr, g, nnz_in, c_in, c_out, g_rows, &w);
    return w.total;
}

int sparse_conv_bwd(int ndim, const int32_t* extent, int batch, const int32_t* in_coords, const float* in_feats,
                    int64_t nnz_in, int c_in, const int32_t* ksize, const float* w, int c_out,
                    const int32_t* g_coords, const float* g_feats, int64_t g_rows, float* bp_data, float* bp_filter,
                    int64_t* info, void* workspace, size_t workspace_bytes, void* hip_stream) {
    Geom g;
    if (!ksize) return fail(SCNN_EINVAL, "ksize is null");
    int rc = make_geom(ndim, extent, batch, ksize, &g);
    if (rc != SCNN_OK) return rc;
    rc = check_bwd_sizes(g, nnz_in, c_in, c_out, g_rows);
    if (rc != SCNN_OK) return rc;
    if (!w || !bp_filter || !info || !workspace) return fail(SCNN_EINVAL, "null pointer (w, bp_filter, info or workspace)");
    if (nnz_in > 0 && (!in_coords || !in_feats || !bp_data)) return fail(SCNN_EINVAL, "null input arrays");
    if (g_rows > 0 && (!g_coords || !g_feats)) return fail(SCNN_EINVAL, "null gradient arrays");
    if (((uintptr_t)workspace & 255) != 0) return fail(SCNN_EWORKSPACE, "workspace must be 256-byte aligned");
    BwdWs ws;
    carve_bwd(workspace, g, nnz_in, c_in, c_out, g_rows, &ws);
    if (ws.total > workspace_bytes)
        return fail(SCNN_EWORKSPACE, "workspace too small: %zu < %zu bytes", workspace_bytes, ws.total);
    hipStream_t s = (hipStream_t)hip_stream;
    const long long n_elem = (long long)g.T * c_in * c_out;
    const bool use_mfma = g_conv_path != 1 && ws.mfma_shape && nnz_in > 0 && ((uintptr_t)in_feats & 15) == 0 &&
                          ((uintptr_t)g_feats & 15) == 0;
    const int n_chunks = use_mfma ? ws.chunks_mfma : ws.chunks_valu;

    StageTimer timer(s, kFwdStages, kBwdStages);
    timer.mark();
    // adjoint filter (taps negated, channels transposed) in the layout of the convolution kernel that will run;
    // the same launch clears the counters and the occupancy bitmap
    SCNN_TRY(launch_prepare(g, w, c_out, c_in, 1, ws.c_in_pad, ws.wp, use_mfma ? ws.wb : nullptr, nullptr,
                            ws.tap_active, ws.tap_coord, workspace, ws.zero_bytes, s));
    SCNN_TRY(launch_index_build(g, g_coords, g_rows, nullptr, g_rows, ws.occ, ws.occ_prefix, ws.ctr, s));
    SCNN_TRY(launch_rows_sample_bounds(g, in_coords, nnz_in, ws.cand_start, ws.tile_start, ws.ctr, s));
    SCNN_TRY(launch_bwd_sites(g, in_coords, nnz_in, ws.cand_start, ws.cand_lin, ws.rows16_start, ws.ctr, s));
    timer.mark();
    if (use_mfma) {
        SCNN_TRY(launch_pair_build(g, ws.occ, ws.occ_prefix, g_rows, ws.tap_active, ws.tap_coord, ws.cand_lin,
                                   ws.cand_start, ws.tile_start, ws.rows16_start, ws.ctr, ws.pairs, ws.block_tap,
                                   ws.tile_hdr, ws.block_cap, ws.tiles_cap, ws.tap_first, s));
        timer.mark();
        SCNN_TRY(launch_conv_mfma(g, g_rows, g_feats, c_out, ws.wb, c_in, nullptr, ws.pairs, ws.block_tap,
                                  ws.tile_hdr, ws.ctr, ws.resp, s));
    } else {
        timer.mark();
        SCNN_TRY(launch_conv_valu(g, ws.occ, ws.occ_prefix, g_rows, g_feats, c_out, ws.wp, c_in, ws.c_in_pad, nullptr,
                                  ws.tap_active, ws.cand_lin, ws.cand_start, ws.tile_start, ws.ctr, ws.tiles_cap,
                                  ws.resp, s));
    }
    timer.mark();
    SCNN_TRY(launch_bwd_data_write(g, ws.resp, in_feats, c_in, ws.cand_start, ws.tile_start, ws.ctr, ws.tiles_cap,
                                   bp_data, s));
    timer.mark();
    if (use_mfma)
        SCNN_TRY(launch_bwd_filter_mfma(g, in_feats, c_in, g_feats, c_out, ws.pairs, ws.tap_first, ws.tile_hdr,
                                        ws.cand_start, ws.tile_start, ws.ctr, n_chunks, ws.fpart, s));
    else
        SCNN_TRY(launch_bwd_filter_valu(g, ws.occ, ws.occ_prefix, g_rows, g_feats, c_out, in_feats, c_in,
                                        ws.tap_active, ws.cand_lin, ws.cand_start, ws.tile_start, ws.ctr, n_chunks,
                                        ws.fpart, s));
    SCNN_TRY(launch_bwd_filter_finish(ws.fpart, n_chunks, n_elem, w, bp_filter, ws.ctr, nnz_in, g_rows,
                                      (long long*)info, s));
    timer.done();
    return SCNN_OK;
}

int sparse_conv_fwd(int ndim, const int32_t* extent, int batch, const int32_t* in_coords, const float* in_feats,
                    int64_t nnz_in, int c_in, const int32_t* ksize, const float* w, const float* bias, int c_out,
                    double rho_up, int topk_mode, unsigned fuse, int32_t* out_coords, float* out_feats,
                    int64_t out_capacity, int64_t cand_capacity, int64_t* nnz_out, void* workspace,
                    size_t workspace_bytes, void* hip_stream) {
    return conv_fwd_impl(ndim, extent, batch, in_coords, in_feats, nnz_in, nullptr, c_in, ksize, w, bias, c_out, rho_up,
                         topk_mode, fuse, out_coords, out_feats, out_capacity, cand_capacity, nnz_out, workspace,
                         workspace_bytes, hip_stream);
}

int sparse_conv_fwd_chained(int ndim, const int32_t* extent, int batch, const int32_t* in_coords,
                            const float* in_feats, int64_t in_capacity, const int64_t* nnz_in_dev, int c_in,
                            const int32_t* ksize, const float* w, const float* bias, int c_out, double rho_up,
                            int topk_mode, unsigned fuse, int32_t* out_coords, float* out_feats, int64_t out_capacity,
                            int64_t cand_capacity, int64_t* nnz_out, void* workspace, size_t workspace_bytes,
                            void* hip_stream) {
    if (!nnz_in_dev) return fail(SCNN_EINVAL, "nnz_in_dev is null");
    return conv_fwd_impl(ndim, extent, batch, in_coords, in_feats, in_capacity, nnz_in_dev, c_in, ksize, w, bias, c_out,
                         rho_up, topk_mode, fuse, out_coords, out_feats, out_capacity, cand_capacity, nnz_out,
                         workspace, workspace_bytes, hip_stream);
}

int scnn_set_conv_path(int path) {
    if (path < 0 || path > 3)
        return fail(SCNN_EINVAL, "conv path must be 0 (auto), 1 (vector kernels), 2 (matrix cores where possible) or 3 (pair-list matrix-core kernel)");
    g_conv_path = path;
    return SCNN_OK;
}

const char* scnn_last_conv_kernel(void) { return g_last_conv_kernel; }

int scnn_calibration_copy(void* dst, const void* src, size_t bytes, void* hip_stream) {
    if (!dst || !src || bytes % 16 != 0) return fail(SCNN_EINVAL, "calibration copy needs non-null pointers and a multiple of 16 bytes");
    SCNN_TRY(launch_calibration_copy(dst, src, bytes, (hipStream_t)hip_stream));
    return SCNN_OK;
}

int scnn_profile_enable(int on) {
    if (on < 0 || on > 3) return fail(SCNN_EINVAL, "profile mode must be 0, 1, 2 or 3");
    g_prof_on = on;
    g_prof_tick = 0;
    return SCNN_OK;
}

int scnn_profile_stage_count(void) { return kStages; }

const char* scnn_profile_stage_name(int i) { return (i >= 0 && i < kStages) ? kStageNames[i] : ""; }

int scnn_profile_collect(double* stage_ms, int64_t* calls) {
    if (!stage_ms || !calls) return fail(SCNN_EINVAL, "null pointer");
    for (int i = 0; i < kStages; ++i) stage_ms[i] = 0.0;
    *calls = 0;
    if (!g_prof_calls) return SCNN_OK;
    for (ProfCall& c : *g_prof_calls) {
        for (int i = c.n_stages; i >= 0; --i)
            if (c.recorded >> i & 1u) {
                SCNN_TRY(hipEventSynchronize(c.ev[i]));  // the call's last recorded event
                break;
            }
        for (int i = 0; i < c.n_stages; ++i) {
            if ((c.recorded >> i & 3u) != 3u) continue;  // a stage needs both of its boundaries
            float ms = 0.0f;
            SCNN_TRY(hipEventElapsedTime(&ms, c.ev[i], c.ev[i + 1]));
            stage_ms[c.first_stage + i] += (double)ms;
        }
        ++*calls;
        g_prof_pool->push_back(c);
    }
    g_prof_calls->clear();
    return SCNN_OK;
}

// ---------------------------------------------------------------- attention_topk
namespace {
struct TopkWs {
    Counters* ctr;
    ColState* cols;
    unsigned long long* tile_state;
    size_t zero_bytes;
    uint2* part;
    unsigned long long* row_keep;
    unsigned long long* row_plane;
    long long* tile_base;
    bool marks;
    unsigned* block_sums;
    int* cand_start;
    int* tile_start;
    unsigned* cand_lin;
    float* resp;
    uint2* side;
    unsigned long long side_cap;
    long long tiles_cap;
    size_t total;
};
void carve_topk(void* base, const Geom& g, long long rows, int channels, TopkWs* w) {
    Carver c(base);
    const long long ncols = (long long)g.batch * channels;
    w->tiles_cap = (rows + kTileRows - 1) / kTileRows + g.batch;
    w->ctr = c.take<Counters>(1);
    w->marks = !topk_small_columns(g) && channels > kMarkMinChannels && channels <= kMarkPlanes;
    w->cols = c.take<ColState>(ncols);
    w->tile_state = c.take<unsigned long long>(w->tiles_cap);
    w->zero_bytes = c.total();
    w->part = c.take<uint2>(topk_small_columns(g) ? 0 : ncols * kTopkPartWords);
    w->row_keep = c.take<unsigned long long>(w->marks ? 2 * w->tiles_cap : 0);
    w->row_plane = c.take<unsigned long long>(w->marks ? 2 * w->tiles_cap * kMarkPlanes : 0);
    w->tile_base = c.take<long long>(w->marks ? w->tiles_cap : 0);
    w->block_sums = c.take<unsigned>(scan_blocks(w->tiles_cap));
    w->cand_start = c.take<int>(g.batch + 1);
    w->tile_start = c.take<int>(g.batch + 1);
    w->cand_lin = c.take<unsigned>(rows > 0 ? rows : 1);
    w->resp = c.take<float>((size_t)w->tiles_cap * channels * kTileRows);
    w->side_cap = (unsigned long long)w->tiles_cap * kTileRows * channels;
    w->side = c.take<uint2>((size_t)w->side_cap);
    w->total = c.total();
}
}  // namespace

size_t attention_topk_workspace(int ndim, const int32_t* extent, int batch, int64_t rows, int channels) {
    Geom g;
    if (make_geom(ndim, extent, batch, nullptr, &g) != SCNN_OK) return 0;
    if (rows < 0 || rows > kMaxIndex - (long long)batch * kTileRows || channels < 1 || channels > kMaxChannels) return 0;
    TopkWs w;
    carve_topk(nullptr, g, rows, channels, &w);
    return w.total;
}

int attention_topk(int ndim, const int32_t* extent, int batch, const int32_t* coords, const float* resp,
                   int64_t rows, int channels, int64_t k, int topk_mode, int32_t* out_coords, float* out_feats,
                   int64_t out_capacity, int64_t* nnz_out, void* workspace, size_t workspace_bytes, void* hip_stream) {
    Geom g;
    int rc = make_geom(ndim, extent, batch, nullptr, &g);
    if (rc != SCNN_OK) return rc;
    if (rows < 0 || rows > kMaxIndex - (long long)batch * kTileRows) return fail(SCNN_ECAPACITY, "rows out of range");
    if (channels < 1) return fail(SCNN_EINVAL, "channels must be positive");
    if (channels > kMaxChannels) return fail(SCNN_ECAPACITY, "at most %d channels", kMaxChannels);
    if (k < 0) return fail(SCNN_EINVAL, "k < 0");
    if (topk_mode != SCNN_TOPK_ABS && topk_mode != SCNN_TOPK_SIGNED) return fail(SCNN_EINVAL, "bad topk_mode");
    if (!nnz_out || !workspace) return fail(SCNN_EINVAL, "null pointer (nnz_out or workspace)");
    if (rows > 0 && (!coords || !resp)) return fail(SCNN_EINVAL, "null input arrays");
    if (out_capacity < 0 || out_capacity > kMaxIndex) return fail(SCNN_EINVAL, "bad out_capacity");
    if (out_capacity > 0 && (!out_coords || !out_feats)) return fail(SCNN_EINVAL, "null output arrays");
    if (((uintptr_t)workspace & 255) != 0) return fail(SCNN_EWORKSPACE, "workspace must be 256-byte aligned");
    TopkWs ws;
    carve_topk(workspace, g, rows, channels, &ws);
    if (ws.total > workspace_bytes)
        return fail(SCNN_EWORKSPACE, "workspace too small: %zu < %zu bytes", workspace_bytes, ws.total);
    hipStream_t s = (hipStream_t)hip_stream;
    SCNN_TRY(launch_zero(workspace, ws.zero_bytes, s));
    SCNN_TRY(launch_rows_sample_bounds(g, coords, rows, ws.cand_start, ws.tile_start, ws.ctr, s));
    SCNN_TRY(launch_rows_to_planar(g, coords, resp, channels, ws.cand_start, ws.tile_start, ws.ctr, ws.tiles_cap,
                                   ws.cand_lin, ws.resp, s));
    const bool marks = ws.marks && k > 0;
    SCNN_TRY(launch_topk(g, channels, k, topk_mode, 0, ws.tile_start, ws.resp, ws.cols, ws.side, ws.part,
                         marks ? ws.row_keep : nullptr, marks ? ws.row_plane : nullptr, marks ? ws.tile_base : nullptr,
                         ws.tiles_cap, ws.ctr, s));
    SCNN_TRY(launch_select_write(g, channels, topk_mode, 0, ws.cand_start, ws.tile_start, ws.cand_lin, ws.resp,
                                 ws.cols, ws.tile_state, ws.tiles_cap, ws.ctr, out_coords, out_feats, out_capacity,
                                 (long long*)nnz_out, rows, 0, marks ? ws.tile_base : nullptr, s));
    return SCNN_OK;
}

// ---------------------------------------------------------------- sparse_relu
size_t sparse_relu_workspace(int64_t rows, int channels) {
    if (rows < 0 || rows > kMaxIndex || channels < 1) return 0;
    Carver c(nullptr);
    c.take<Counters>(1);
    c.take<unsigned>(rows > 0 ? rows : 1);
    c.take<unsigned>(rows > 0 ? rows : 1);
    c.take<unsigned>(scan_blocks(rows));
    return c.total();
}

int sparse_relu(int ndim, const int32_t* coords, const float* feats, int64_t rows, int channels,
                int32_t* out_coords, float* out_feats, int64_t out_capacity, int64_t* nnz_out, void* workspace,
                size_t workspace_bytes, void* hip_stream) {
    if (ndim != 2 && ndim != 3) return fail(SCNN_EINVAL, "ndim must be 2 or 3 (got %d)", ndim);
    if (rows < 0 || rows > kMaxIndex) return fail(SCNN_ECAPACITY, "rows out of range");
    if (channels < 1) return fail(SCNN_EINVAL, "channels must be positive");
    if (!nnz_out || !workspace) return fail(SCNN_EINVAL, "null pointer (nnz_out or workspace)");
    if (rows > 0 && (!coords || !feats)) return fail(SCNN_EINVAL, "null input arrays");
    if (out_capacity < 0 || out_capacity > kMaxIndex) return fail(SCNN_EINVAL, "bad out_capacity");
    if (out_capacity > 0 && (!out_coords || !out_feats)) return fail(SCNN_EINVAL, "null output arrays");
    if (((uintptr_t)workspace & 255) != 0) return fail(SCNN_EWORKSPACE, "workspace must be 256-byte aligned");
    Carver c(workspace);
    Counters* ctr = c.take<Counters>(1);
    const size_t zero_bytes = c.total();
    unsigned* flags = c.take<unsigned>(rows > 0 ? rows : 1);
    unsigned* offs = c.take<unsigned>(rows > 0 ? rows : 1);
    unsigned* block_sums = c.take<unsigned>(scan_blocks(rows));
    if (c.total() > workspace_bytes)
        return fail(SCNN_EWORKSPACE, "workspace too small: %zu < %zu bytes", workspace_bytes, c.total());
    Geom g;
    memset(&g, 0, sizeof(g));
    g.ndim = ndim;
    hipStream_t s = (hipStream_t)hip_stream;
    SCNN_TRY(launch_zero(workspace, zero_bytes, s));
    SCNN_TRY(launch_relu(g, coords, feats, rows, channels, flags, offs, block_sums, out_coords, out_feats,
                         out_capacity, ctr, s));
    SCNN_TRY(launch_finish(ctr, 0, rows, 0, out_capacity, (long long*)nnz_out, s));
    return SCNN_OK;
}

// ---------------------------------------------------------------- sparse_relu without a workspace
// The same kernels as sparse_relu; the counters, row flags, row offsets and scan sums live in a device array
// that is part of the library image instead of a caller's workspace.  Each GPU holds its own copy of the array at
// its own address: the address is looked up once per device, with that device current, and only that address
// (never the array's name) is handed to kernels.
namespace {
constexpr long long kStaticReluMaxRows = 1ll << 20;
constexpr size_t kStaticReluBytes = (sizeof(Counters) + 255) / 256 * 256                     // Counters
                                    + 2 * (size_t)kStaticReluMaxRows * sizeof(unsigned)      // flags, offsets
                                    + (((size_t)kStaticReluMaxRows / kScanChunk + 2) * sizeof(unsigned) + 255) / 256 * 256;
constexpr int kMaxDevices = 64;
}  // namespace
static __device__ __align__(256) unsigned char scratch[kStaticReluBytes];
namespace {
void* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

// Device address of `scratch` on the current device (looked up on the first call per device).
int static_scratch(void** out) {
    int dev = -1;
    SCNN_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(SCNN_ECAPACITY, "device ordinal %d not supported (at most %d)", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        SCNN_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p || ((uintptr_t)p & 255) != 0) return fail(SCNN_EHIP, "static scratch array has no usable device address");
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return SCNN_OK;
}
}  // namespace

int64_t sparse_relu_static_max_rows(void) { return kStaticReluMaxRows; }

int sparse_relu_static(int ndim, const int32_t* coords, const float* feats, int64_t rows, int channels,
                       int32_t* out_coords, float* out_feats, int64_t out_capacity, int64_t* nnz_out,
                       void* hip_stream) {
    if (ndim != 2 && ndim != 3) return fail(SCNN_EINVAL, "ndim must be 2 or 3 (got %d)", ndim);
    if (rows < 0) return fail(SCNN_EINVAL, "rows < 0");
    if (rows > kStaticReluMaxRows)
        return fail(SCNN_ECAPACITY, "sparse_relu_static takes at most %lld rows (got %lld): use sparse_relu with a workspace",
                    kStaticReluMaxRows, (long long)rows);
    if (channels < 1) return fail(SCNN_EINVAL, "channels must be positive");
    if (channels > kMaxChannels) return fail(SCNN_ECAPACITY, "at most %d channels", kMaxChannels);
    if (!nnz_out) return fail(SCNN_EINVAL, "nnz_out is null");
    if (rows > 0 && (!coords || !feats)) return fail(SCNN_EINVAL, "null input arrays");
    if (out_capacity < 0 || out_capacity > kMaxIndex) return fail(SCNN_EINVAL, "bad out_capacity");
    if (out_capacity > 0 && (!out_coords || !out_feats)) return fail(SCNN_EINVAL, "null output arrays");
    void* base = nullptr;
    int rc = static_scratch(&base);
    if (rc != SCNN_OK) return rc;
    Carver c(base);
    Counters* ctr = c.take<Counters>(1);
    const size_t zero_bytes = c.total();
    unsigned* flags = c.take<unsigned>(kStaticReluMaxRows);
    unsigned* offs = c.take<unsigned>(kStaticReluMaxRows);
    unsigned* block_sums = c.take<unsigned>(scan_blocks(kStaticReluMaxRows));
    if (c.total() > kStaticReluBytes) return fail(SCNN_EWORKSPACE, "static scratch layout exceeds the array");
    Geom g;
    memset(&g, 0, sizeof(g));
    g.ndim = ndim;
    hipStream_t s = (hipStream_t)hip_stream;
    // the array keeps the previous call's contents: the counters start from zero through a fill kernel (no memset
    // node, so the call can be captured); flags and offsets of rows [0, rows) are rewritten before they are read
    SCNN_TRY(launch_zero(base, zero_bytes, s));
    SCNN_TRY(launch_relu(g, coords, feats, rows, channels, flags, offs, block_sums, out_coords, out_feats,
                         out_capacity, ctr, s));
    SCNN_TRY(launch_finish(ctr, 0, rows, 0, out_capacity, (long long*)nnz_out, s));
    return SCNN_OK;
}

// ---------------------------------------------------------------- sparse_maxpool
namespace {
struct PoolWs {
    Counters* ctr;
    unsigned long long* occ;
    unsigned long long* pbits;
    size_t zero_bytes;
    unsigned* occ_prefix;
    unsigned* pprefix;
    unsigned* block_sums;
    long long* pool_key;
    long long pool_cap;
    size_t total;
};
void carve_pool(void* base, const Geom& g, const Geom& gp, long long rows, PoolWs* w) {
    Carver c(base);
    const long long nw = (long long)g.batch * g.Wps, nwp = (long long)gp.batch * gp.Wps;
    const long long grid_p = (long long)gp.batch * gp.N;
    w->pool_cap = rows < grid_p ? rows : grid_p;
    if (w->pool_cap < 1) w->pool_cap = 1;
    w->ctr = c.take<Counters>(1);
    w->occ = c.take<unsigned long long>(nw);
    w->pbits = c.take<unsigned long long>(nwp);
    w->zero_bytes = c.total();
    w->occ_prefix = c.take<unsigned>(nw);
    w->pprefix = c.take<unsigned>(nwp);
    // (up to kEmitMidWords words the pooling keeps a count per chunk of 256 words instead of the scan's sums)
    w->block_sums = c.take<unsigned>(nwp <= kEmitMidWords && (nwp + 255) / 256 > scan_blocks(nwp) ? (nwp + 255) / 256
                                                                                                  : scan_blocks(nwp));
    w->pool_key = c.take<long long>(w->pool_cap);
    w->total = c.total();
}
}  // namespace

size_t sparse_maxpool_workspace(int ndim, const int32_t* extent, int batch, int64_t rows, int channels) {
    Geom g;
    if (make_geom(ndim, extent, batch, nullptr, &g) != SCNN_OK) return 0;
    if (rows < 0 || rows > kMaxIndex || channels < 1) return 0;
    PoolWs w;
    carve_pool(nullptr, g, pooled_geom(g), rows, &w);
    return w.total;
}

int sparse_maxpool(int ndim, const int32_t* extent, int batch, int window, const int32_t* coords, const float* feats,
                   int64_t rows, int channels, int32_t* out_coords, float* out_feats, int64_t out_capacity,
                   int64_t* nnz_out, void* workspace, size_t workspace_bytes, void* hip_stream) {
    Geom g;
    int rc = make_geom(ndim, extent, batch, nullptr, &g);
    if (rc != SCNN_OK) return rc;
    if (window != 2) return fail(SCNN_EINVAL, "only window = stride = 2 is implemented (got %d)", window);
    if (rows < 0 || rows > kMaxIndex) return fail(SCNN_ECAPACITY, "rows out of range");
    if (channels < 1) return fail(SCNN_EINVAL, "channels must be positive");
    if (!nnz_out || !workspace) return fail(SCNN_EINVAL, "null pointer (nnz_out or workspace)");
    if (rows > 0 && (!coords || !feats)) return fail(SCNN_EINVAL, "null input arrays");
    if (out_capacity < 0 || out_capacity > kMaxIndex) return fail(SCNN_EINVAL, "bad out_capacity");
    if (out_capacity > 0 && (!out_coords || !out_feats)) return fail(SCNN_EINVAL, "null output arrays");
    if (((uintptr_t)workspace & 255) != 0) return fail(SCNN_EWORKSPACE, "workspace must be 256-byte aligned");
    const Geom gp = pooled_geom(g);
    PoolWs ws;
    carve_pool(workspace, g, gp, rows, &ws);
    if (ws.total > workspace_bytes)
        return fail(SCNN_EWORKSPACE, "workspace too small: %zu < %zu bytes", workspace_bytes, ws.total);
    hipStream_t s = (hipStream_t)hip_stream;
    SCNN_TRY(launch_zero(workspace, ws.zero_bytes, s));
    SCNN_TRY(launch_maxpool(g, gp, coords, feats, rows, nullptr, rows, channels, 0, ws.occ, ws.occ_prefix, ws.pbits,
                            ws.pprefix, ws.block_sums, ws.pool_key, ws.pool_cap, out_coords, out_feats, out_capacity,
                            ws.ctr, (long long*)nnz_out, rows, 0, s));
    return SCNN_OK;
}

// ---------------------------------------------------------------- sparse_to_dense
int sparse_to_dense(int ndim, const int32_t* extent, int batch, const int32_t* coords, const float* feats,
                    int64_t rows, const int64_t* rows_dev, int channels, float* dense, void* hip_stream) {
    Geom g;
    int rc = make_geom(ndim, extent, batch, nullptr, &g);
    if (rc != SCNN_OK) return rc;
    if (rows < 0 || rows > kMaxIndex) return fail(SCNN_ECAPACITY, "rows out of range");
    if (channels < 1) return fail(SCNN_EINVAL, "channels must be positive");
    if (channels > kMaxChannels) return fail(SCNN_ECAPACITY, "at most %d channels", kMaxChannels);
    if (!dense) return fail(SCNN_EINVAL, "dense is null");
    if (((uintptr_t)dense & 15) != 0) return fail(SCNN_EINVAL, "dense must be 16-byte aligned");
    if (rows > 0 && (!coords || !feats)) return fail(SCNN_EINVAL, "null input arrays");
    SCNN_TRY(launch_to_dense(g, coords, feats, rows, (const long long*)rows_dev, channels, dense, (hipStream_t)hip_stream));
    return SCNN_OK;
}

// ---------------------------------------------------------------- regulariser and pruning
size_t density_regulariser_workspace(void) { return 256 + 256 * sizeof(double); }

int density_regulariser(const float* out_feats, int64_t rows, const int64_t* rows_dev, int channels, int64_t n_sites_total,
                        double rho_up, double o, double b1, double b2, double lambda, const float* w, int64_t n_w,
                        float* grad_w, double* result, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (rows < 0 || rows > kMaxIndex) return fail(SCNN_ECAPACITY, "rows out of range");
    if (channels < 1 || channels > kMaxChannels) return fail(SCNN_EINVAL, "bad channel count");
    if (n_sites_total < 1) return fail(SCNN_EINVAL, "n_sites_total must be positive");
    if (!(rho_up >= 0.0 && rho_up <= 1.0)) return fail(SCNN_EINVAL, "rho_up = %g not in [0, 1]", rho_up);
    if (!(o >= 0.0) || !(b1 >= 0.0) || !(b2 >= 0.0)) return fail(SCNN_EINVAL, "o, b1, b2 must be >= 0");
    if (n_w < 0 || n_w > kMaxIndex) return fail(SCNN_ECAPACITY, "n_w out of range");
    if (!result || !workspace || (n_w > 0 && !w)) return fail(SCNN_EINVAL, "null pointer");
    if (rows > 0 && !out_feats) return fail(SCNN_EINVAL, "null out_feats");
    if (((uintptr_t)workspace & 255) != 0 || workspace_bytes < density_regulariser_workspace())
        return fail(SCNN_EWORKSPACE, "workspace too small or misaligned");
    unsigned long long* count = (unsigned long long*)workspace;
    double* partial = (double*)((char*)workspace + 256);
    SCNN_TRY(launch_density_regulariser(out_feats, rows, (const long long*)rows_dev, rows, channels,
                                        (double)n_sites_total * channels, rho_up, o, b1, b2, lambda, w, n_w, grad_w,
                                        count, partial, result, (hipStream_t)hip_stream));
    return SCNN_OK;
}

int prune_weights(float* w, unsigned char* warned, int64_t n_w, float eps, int64_t* counts, void* hip_stream) {
    if (n_w < 0 || n_w > kMaxIndex) return fail(SCNN_ECAPACITY, "n_w out of range");
    if (!(eps >= 0.0f)) return fail(SCNN_EINVAL, "eps must be >= 0");
    if (!counts || (n_w > 0 && (!w || !warned))) return fail(SCNN_EINVAL, "null pointer");
    SCNN_TRY(launch_prune(w, warned, n_w, eps, (unsigned long long*)counts, (hipStream_t)hip_stream));
    return SCNN_OK;
}

// ---------------------------------------------------------------- validation
int scnn_validate_rows(int ndim, const int32_t* extent, int batch, const int32_t* coords, int64_t rows,
                       void* workspace, size_t workspace_bytes, void* hip_stream) {
    Geom g;
    int rc = make_geom(ndim, extent, batch, nullptr, &g);
    if (rc != SCNN_OK) return rc;
    if (rows < 0 || rows > kMaxIndex) return fail(SCNN_ECAPACITY, "rows out of range");
    if (rows == 0) return SCNN_OK;
    if (!coords || !workspace) return fail(SCNN_EINVAL, "null pointer");
    if (workspace_bytes < 256 || ((uintptr_t)workspace & 255) != 0) return fail(SCNN_EWORKSPACE, "need 256 aligned bytes");
    hipStream_t s = (hipStream_t)hip_stream;
    Counters* ctr = (Counters*)workspace;
    // (the check only touches the status bits, which sit in the first 256 bytes of the counters)
    static_assert(offsetof(Counters, flags) + sizeof(unsigned) <= 256, "status bits within the documented workspace");
    SCNN_TRY(launch_zero(workspace, 256, s));
    SCNN_TRY(launch_validate(g, coords, rows, ctr, s));
    struct { unsigned flags; } host;
    SCNN_TRY(hipMemcpyAsync(&host.flags, &ctr->flags, sizeof(unsigned), hipMemcpyDeviceToHost, s));
    SCNN_TRY(hipStreamSynchronize(s));
    if (host.flags & SCNN_FLAG_BAD_COORD) return fail(SCNN_EINVAL, "a coordinate lies outside the grid");
    if (host.flags & SCNN_FLAG_UNSORTED) return fail(SCNN_EUNSORTED, "rows are not strictly ascending by (b, lin)");
    return SCNN_OK;
}

}  // extern "C"
