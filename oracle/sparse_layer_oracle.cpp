// CPU oracle for the forward direct sparse convolution layer with attention.
//
// THIS FILE IS TEST INFRASTRUCTURE.  It is a slow, literal, single-file CPU
// statement of what the layer computes, written from the paper (Hackel et al.,
// "Inference, Learning and Attention Mechanisms that Exploit and Preserve
// Sparsity in CNNs"): Algorithm 1 (direct sparse convolution with attention),
// Sec. 3.2 (k-selection on each output channel), Sec. 3.3 (pooling: rewrite
// keys, sort, reduce each cluster), Algorithm 2 with Eq. 3 (back-propagation
// to non-zero inputs and un-pruned weights only).  It shares no code with the HIP library
// and must never be called from the product path: only the tests, the smoke
// check and the benchmark's CPU-baseline leg use it.
//
// Conventions (the paper leaves these open; the same readings are used by the
// HIP library and are listed in the design notes):
//   * site index lin = row-major over the d spatial coordinates, last fastest;
//   * filter tap index t = row-major over (delta_1..delta_d) + h, h=(s_f-1)/2;
//   * get_update_id (Alg. 1 step 8): an input at site q hit through tap delta
//     updates output site p = q - delta (cross-correlation with zero "same"
//     padding, stride 1); updates that leave the grid are dropped;
//   * accumulation in double, one rounding to float per site (Alg. 1 step 9);
//   * "non-zero entries" (step 13) = sites whose float value != 0;
//   * bias (step 14) is one scalar per output channel, added to those entries;
//     an entry whose biased value is exactly 0 is not a candidate any more;
//   * k-selection (step 15) is per (sample, output channel): keep the first
//     min(k, count) candidates in the order (score descending, lin ascending);
//     score = |v| (mode 0) or v (mode 1);
//   * sparse ReLU keeps entries with v > 0;
//   * max-pooling: window = stride = 2 per spatial axis, output site floor(p/2),
//     output extent ceil(E/2), maximum over the *present* entries of a cluster;
//   * a row of the output = a site with at least one surviving entry; absent
//     entries of a row are stored as 0.0f; rows ascend by (b, lin).
//
// Build: g++ -O2 -std=c++17 -fopenmp -shared -fPIC (no fast-math).
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>
#ifdef _OPENMP
#include <omp.h>
#endif

namespace {

struct Entry {
    int32_t b;
    int64_t lin;
    int32_t c;
    float v;
};

struct Geometry {
    int ndim;
    int64_t extent[3];
    int64_t n_sites;  // N = prod(extent)
};

struct Result {
    int ndim = 0;
    int channels = 0;
    std::vector<int32_t> coords;  // [rows, 1+ndim]
    std::vector<float> feats;     // [rows, channels]
    int64_t rows = 0;
    int64_t macs = 0;       // multiply-adds executed by the conv loop nest
    int threads_used = 1;
};

Result g_result;

Geometry make_geometry(int ndim, const int32_t* extent) {
    Geometry g;
    g.ndim = ndim;
    g.n_sites = 1;
    for (int a = 0; a < 3; ++a) g.extent[a] = 1;
    for (int a = 0; a < ndim; ++a) {
        g.extent[a] = extent[a];
        g.n_sites *= extent[a];
    }
    return g;
}

int64_t lin_of(const Geometry& g, const int64_t* p) {
    int64_t lin = 0;
    for (int a = 0; a < g.ndim; ++a) lin = lin * g.extent[a] + p[a];
    return lin;
}

void site_of(const Geometry& g, int64_t lin, int64_t* p) {
    for (int a = g.ndim - 1; a >= 0; --a) {
        p[a] = lin % g.extent[a];
        lin /= g.extent[a];
    }
}

// Sec. 3.2: the selection keeps "the k strongest (non-zero) responses".
// Written as the plain definition: sort all candidates, take the first k.
void select_k(std::vector<std::pair<float, int64_t>>& cand /* (value, lin) */, int64_t k, int mode,
              std::vector<std::pair<float, int64_t>>& kept) {
    auto score = [mode](float v) { return mode == 0 ? std::fabs(v) : v; };
    std::stable_sort(cand.begin(), cand.end(),
                     [&](const std::pair<float, int64_t>& x, const std::pair<float, int64_t>& y) {
                         float sx = score(x.first), sy = score(y.first);
                         if (sx != sy) return sx > sy;
                         return x.second < y.second;
                     });
    int64_t n = std::min<int64_t>(k, (int64_t)cand.size());
    if (n < 0) n = 0;
    kept.assign(cand.begin(), cand.begin() + n);
}

// entries -> rows sorted by (b, lin); absent channel entries are 0.0f.
void assemble_rows(std::vector<Entry>& e, const Geometry& g, int channels, Result& r) {
    std::sort(e.begin(), e.end(), [](const Entry& x, const Entry& y) {
        if (x.b != y.b) return x.b < y.b;
        if (x.lin != y.lin) return x.lin < y.lin;
        return x.c < y.c;
    });
    r.ndim = g.ndim;
    r.channels = channels;
    r.coords.clear();
    r.feats.clear();
    r.rows = 0;
    size_t i = 0;
    while (i < e.size()) {
        size_t j = i;
        int64_t p[3];
        site_of(g, e[i].lin, p);
        r.coords.push_back(e[i].b);
        for (int a = 0; a < g.ndim; ++a) r.coords.push_back((int32_t)p[a]);
        size_t base = r.feats.size();
        r.feats.resize(base + channels, 0.0f);
        while (j < e.size() && e[j].b == e[i].b && e[j].lin == e[i].lin) {
            r.feats[base + e[j].c] = e[j].v;
            ++j;
        }
        ++r.rows;
        i = j;
    }
}

void rows_to_entries(const Geometry& g, const int32_t* coords, const float* feats, int64_t rows, int channels,
                     std::vector<Entry>& e) {
    e.clear();
    for (int64_t r = 0; r < rows; ++r) {
        const int32_t* c = coords + r * (1 + g.ndim);
        int64_t p[3] = {0, 0, 0};
        for (int a = 0; a < g.ndim; ++a) p[a] = c[1 + a];
        int64_t lin = lin_of(g, p);
        for (int ch = 0; ch < channels; ++ch) {
            float v = feats[r * channels + ch];
            if (v != 0.0f) e.push_back(Entry{c[0], lin, ch, v});
        }
    }
}

// Sparse ReLU: an entry survives iff v > 0.
void relu_entries(std::vector<Entry>& e) {
    e.erase(std::remove_if(e.begin(), e.end(), [](const Entry& x) { return !(x.v > 0.0f); }), e.end());
}

// Sec. 3.3, three stages: (1) divide the spatial index by the stride,
// (2) sort so that responses of one output voxel are adjacent, (3) reduce each
// cluster with max.  Only stored entries take part.
Geometry pool_entries(std::vector<Entry>& e, const Geometry& g) {
    Geometry gp = g;
    gp.n_sites = 1;
    for (int a = 0; a < g.ndim; ++a) {
        gp.extent[a] = (g.extent[a] + 1) / 2;
        gp.n_sites *= gp.extent[a];
    }
    for (Entry& x : e) {  // stage 1
        int64_t p[3];
        site_of(g, x.lin, p);
        for (int a = 0; a < g.ndim; ++a) p[a] /= 2;
        x.lin = lin_of(gp, p);
    }
    std::stable_sort(e.begin(), e.end(), [](const Entry& x, const Entry& y) {  // stage 2
        if (x.b != y.b) return x.b < y.b;
        if (x.lin != y.lin) return x.lin < y.lin;
        return x.c < y.c;
    });
    std::vector<Entry> out;  // stage 3
    size_t i = 0;
    while (i < e.size()) {
        Entry m = e[i];
        size_t j = i + 1;
        while (j < e.size() && e[j].b == m.b && e[j].lin == m.lin && e[j].c == m.c) {
            if (e[j].v > m.v) m.v = e[j].v;
            ++j;
        }
        out.push_back(m);
        i = j;
    }
    e.swap(out);
    return gp;
}

}  // namespace

extern "C" {

// k from the density bound: "at most rho_up" of the N sites of one channel of
// one sample stay non-zero (Sec. 1 / Sec. 3.2; the paper's experiments use
// rho_up = 1/r so that rho_up*N is an integer).  Floor, except that a product
// within 1e-9 relative of an integer counts as that integer.
int64_t oracle_k_from_rho(double rho_up, int64_t n_sites) {
    double x = rho_up * (double)n_sites;
    double rx = std::floor(x + 0.5);
    int64_t k;
    if (std::fabs(x - rx) <= 1e-9 * std::max(1.0, x))
        k = (int64_t)rx;
    else
        k = (int64_t)std::floor(x);
    if (k < 0) k = 0;
    if (k > n_sites) k = n_sites;
    return k;
}

// Algorithm 1, then optional sparse ReLU (fuse bit 0) and 2^d max-pool (fuse
// bit 1).  Returns the number of output rows (kept in an internal buffer; read
// it with oracle_fetch), or a negative value on bad arguments.
// If resp_only != 0 the selection is skipped (all non-zero responses kept).
int64_t oracle_sparse_conv_fwd(int ndim, const int32_t* extent, int batch, const int32_t* in_coords,
                               const float* in_feats, int64_t nnz_in, int c_in, const int32_t* ksize,
                               const float* w, const float* bias, int c_out, int64_t k, int topk_mode,
                               unsigned fuse, int resp_only, int threads) {
    if (ndim < 1 || ndim > 3 || batch < 0 || c_in <= 0 || c_out <= 0) return -1;
    Geometry g = make_geometry(ndim, extent);
    int64_t ks[3] = {1, 1, 1}, h[3] = {0, 0, 0};
    int64_t taps = 1;
    for (int a = 0; a < ndim; ++a) {
        if (ksize[a] <= 0 || ksize[a] % 2 == 0) return -1;
        ks[a] = ksize[a];
        h[a] = (ksize[a] - 1) / 2;
        taps *= ksize[a];
    }
    // Alg. 1 step 1: expand the tap indices to d-dimensional offsets.
    std::vector<int64_t> tap_delta(taps * 3, 0);
    for (int64_t t = 0; t < taps; ++t) {
        int64_t rem = t;
        for (int a = ndim - 1; a >= 0; --a) {
            tap_delta[t * 3 + a] = rem % ks[a] - h[a];
            rem /= ks[a];
        }
    }
    // rows of each sample (input order kept)
    std::vector<std::vector<int64_t>> rows_of(batch);
    for (int64_t r = 0; r < nnz_in; ++r) {
        int32_t b = in_coords[r * (1 + ndim)];
        if (b < 0 || b >= batch) return -1;
        rows_of[b].push_back(r);
    }

    const int64_t pairs = (int64_t)batch * c_out;
    std::vector<std::vector<Entry>> per_pair(pairs);
    int64_t macs = 0;
    int nthreads = threads > 0 ? threads : 1;
#ifdef _OPENMP
    omp_set_num_threads(nthreads);
#else
    nthreads = 1;
#endif
    int used = 1;
#pragma omp parallel reduction(+ : macs)
    {
#ifdef _OPENMP
#pragma omp single
        used = omp_get_num_threads();
#endif
        std::vector<double> buffer(g.n_sites);
        std::vector<std::pair<float, int64_t>> cand, kept;
#pragma omp for schedule(dynamic, 1)
        for (int64_t pair = 0; pair < pairs; ++pair) {
            const int b = (int)(pair / c_out);   // step 2
            const int oc = (int)(pair % c_out);  // step 3
            std::fill(buffer.begin(), buffer.end(), 0.0);  // step 4
            for (int ic = 0; ic < c_in; ++ic) {            // step 5
                for (int64_t r : rows_of[b]) {             // step 6: {id, val} in data(b, ic)
                    const float val = in_feats[r * c_in + ic];
                    if (val == 0.0f) continue;
                    int64_t q[3] = {0, 0, 0};
                    for (int a = 0; a < ndim; ++a) q[a] = in_coords[r * (1 + ndim) + 1 + a];
                    for (int64_t t = 0; t < taps; ++t) {   // step 7: {fid, fval} in filter(oc, ic)
                        const float fval = w[(t * c_in + ic) * c_out + oc];
                        if (fval == 0.0f) continue;
                        int64_t p[3] = {0, 0, 0};          // step 8: get_update_id
                        bool inside = true;
                        for (int a = 0; a < ndim; ++a) {
                            p[a] = q[a] - tap_delta[t * 3 + a];
                            if (p[a] < 0 || p[a] >= g.extent[a]) inside = false;
                        }
                        if (!inside) continue;
                        buffer[lin_of(g, p)] += (double)val * (double)fval;  // step 9
                        ++macs;
                    }
                }
            }
            cand.clear();
            for (int64_t i = 0; i < g.n_sites; ++i) {      // step 13
                float v = (float)buffer[i];
                if (v == 0.0f) continue;
                if (bias) {                                // step 14
                    v = v + bias[oc];
                    if (v == 0.0f) continue;
                }
                cand.emplace_back(v, i);
            }
            if (resp_only)
                kept = cand;
            else
                select_k(cand, k, topk_mode, kept);        // step 15
            std::vector<Entry>& out = per_pair[pair];      // steps 16-17
            out.reserve(kept.size());
            for (auto& kv : kept) out.push_back(Entry{b, kv.second, oc, kv.first});
        }
    }
    std::vector<Entry> all;
    for (auto& v : per_pair) {
        all.insert(all.end(), v.begin(), v.end());
        std::vector<Entry>().swap(v);
    }
    if (fuse & 1u) relu_entries(all);
    Geometry go = g;
    if (fuse & 2u) go = pool_entries(all, g);
    assemble_rows(all, go, c_out, g_result);
    g_result.macs = macs;
    g_result.threads_used = used;
    return g_result.rows;
}

// Sec. 3.2 alone: k-selection per (sample, channel) over the non-zero entries
// of a site-major response matrix resp[rows, channels].
int64_t oracle_attention_topk(int ndim, const int32_t* extent, int batch, const int32_t* coords,
                              const float* resp, int64_t rows, int channels, int64_t k, int topk_mode) {
    if (ndim < 1 || ndim > 3 || channels <= 0) return -1;
    Geometry g = make_geometry(ndim, extent);
    std::vector<Entry> e, all;
    rows_to_entries(g, coords, resp, rows, channels, e);
    std::vector<std::pair<float, int64_t>> cand, kept;
    for (int b = 0; b < batch; ++b)
        for (int c = 0; c < channels; ++c) {
            cand.clear();
            for (const Entry& x : e)
                if (x.b == b && x.c == c) cand.emplace_back(x.v, x.lin);
            select_k(cand, k, topk_mode, kept);
            for (auto& kv : kept) all.push_back(Entry{b, kv.second, c, kv.first});
        }
    assemble_rows(all, g, channels, g_result);
    g_result.macs = 0;
    return g_result.rows;
}

int64_t oracle_sparse_relu(int ndim, const int32_t* extent, const int32_t* coords, const float* feats,
                           int64_t rows, int channels) {
    if (ndim < 1 || ndim > 3 || channels <= 0) return -1;
    Geometry g = make_geometry(ndim, extent);
    std::vector<Entry> e;
    rows_to_entries(g, coords, feats, rows, channels, e);
    relu_entries(e);
    assemble_rows(e, g, channels, g_result);
    g_result.macs = 0;
    return g_result.rows;
}

int64_t oracle_sparse_maxpool(int ndim, const int32_t* extent, const int32_t* coords, const float* feats,
                              int64_t rows, int channels) {
    if (ndim < 1 || ndim > 3 || channels <= 0) return -1;
    Geometry g = make_geometry(ndim, extent);
    std::vector<Entry> e;
    rows_to_entries(g, coords, feats, rows, channels, e);
    Geometry gp = pool_entries(e, g);
    assemble_rows(e, gp, channels, g_result);
    g_result.macs = 0;
    return g_result.rows;
}

// Algorithm 2 (back-propagation through the convolution) with the masks of
// Eq. 3: gradients reach only non-zero input values and non-zero (un-pruned)
// filter weights.  `g_coords`/`g_feats` hold the gradient of the loss with
// respect to the layer's output as sparse rows on the output grid (the same
// grid as the input: stride 1); sites without a row, and zero entries of a
// row, carry no gradient.  bp_data has the shape of in_feats, bp_filter the
// shape of w; both are overwritten.  Sums are carried in double and rounded to
// float once.  Returns the number of multiply-add pairs visited (each visit
// feeds both outputs), or a negative value on bad arguments.
int64_t oracle_sparse_conv_bwd(int ndim, const int32_t* extent, int batch, const int32_t* in_coords,
                               const float* in_feats, int64_t nnz_in, int c_in, const int32_t* ksize,
                               const float* w, int c_out, const int32_t* g_coords, const float* g_feats,
                               int64_t g_rows, float* bp_data, float* bp_filter) {
    if (ndim < 1 || ndim > 3 || batch < 0 || c_in <= 0 || c_out <= 0) return -1;
    Geometry g = make_geometry(ndim, extent);
    int64_t ks[3] = {1, 1, 1}, h[3] = {0, 0, 0};
    int64_t taps = 1;
    for (int a = 0; a < ndim; ++a) {
        if (ksize[a] <= 0 || ksize[a] % 2 == 0) return -1;
        ks[a] = ksize[a];
        h[a] = (ksize[a] - 1) / 2;
        taps *= ksize[a];
    }
    // steps 1-2: both gradient tensors start at zero
    std::vector<double> d_data((size_t)nnz_in * c_in, 0.0);
    std::vector<double> d_filter((size_t)taps * c_in * c_out, 0.0);
    // step 3: tap index -> d-dimensional offset
    std::vector<int64_t> tap_delta(taps * 3, 0);
    for (int64_t t = 0; t < taps; ++t) {
        int64_t rem = t;
        for (int a = ndim - 1; a >= 0; --a) {
            tap_delta[t * 3 + a] = rem % ks[a] - h[a];
            rem /= ks[a];
        }
    }
    for (int64_t r = 0; r < nnz_in; ++r)
        if (in_coords[r * (1 + ndim)] < 0 || in_coords[r * (1 + ndim)] >= batch) return -1;
    for (int64_t r = 0; r < g_rows; ++r) {
        if (g_coords[r * (1 + ndim)] < 0 || g_coords[r * (1 + ndim)] >= batch) return -1;
        for (int a = 0; a < ndim; ++a)
            if (g_coords[r * (1 + ndim) + 1 + a] < 0 || g_coords[r * (1 + ndim) + 1 + a] >= g.extent[a]) return -1;
    }
    int64_t visits = 0;
    std::vector<double> buffer(g.n_sites);
    for (int b = 0; b < batch; ++b) {                      // step 4
        for (int oc = 0; oc < c_out; ++oc) {               // step 5
            std::fill(buffer.begin(), buffer.end(), 0.0);  // step 6: dense buffer <- gradients(b, oc)
            for (int64_t r = 0; r < g_rows; ++r) {
                const int32_t* c = g_coords + r * (1 + ndim);
                if (c[0] != b) continue;
                int64_t p[3] = {0, 0, 0};
                for (int a = 0; a < ndim; ++a) p[a] = c[1 + a];
                buffer[lin_of(g, p)] = (double)g_feats[r * c_out + oc];
            }
            for (int ic = 0; ic < c_in; ++ic) {            // step 7
                for (int64_t r = 0; r < nnz_in; ++r) {     // step 8: {id, val} in data(b, ic)
                    if (in_coords[r * (1 + ndim)] != b) continue;
                    const float val = in_feats[r * c_in + ic];
                    if (val == 0.0f) continue;
                    int64_t q[3] = {0, 0, 0};
                    for (int a = 0; a < ndim; ++a) q[a] = in_coords[r * (1 + ndim) + 1 + a];
                    for (int64_t t = 0; t < taps; ++t) {   // step 9: {fid, fval} in filter(oc, ic)
                        const float fval = w[(t * c_in + ic) * c_out + oc];
                        if (fval == 0.0f) continue;
                        int64_t p[3] = {0, 0, 0};          // step 10: same get_update_id as the forward pass
                        bool inside = true;
                        for (int a = 0; a < ndim; ++a) {
                            p[a] = q[a] - tap_delta[t * 3 + a];
                            if (p[a] < 0 || p[a] >= g.extent[a]) inside = false;
                        }
                        if (!inside) continue;
                        const double grad = buffer[lin_of(g, p)];                 // step 11
                        d_data[(size_t)r * c_in + ic] += grad * (double)fval;     // step 12
                        d_filter[((size_t)t * c_in + ic) * c_out + oc] += grad * (double)val;  // step 13
                        ++visits;
                    }
                }
            }
        }
    }
    for (size_t i = 0; i < d_data.size(); ++i) bp_data[i] = (float)d_data[i];
    for (size_t i = 0; i < d_filter.size(); ++i) bp_filter[i] = (float)d_filter[i];
    return visits;
}

int64_t oracle_result_rows() { return g_result.rows; }
int64_t oracle_result_macs() { return g_result.macs; }
int oracle_result_threads() { return g_result.threads_used; }

void oracle_fetch(int32_t* coords, float* feats) {
    if (!g_result.coords.empty()) std::memcpy(coords, g_result.coords.data(), g_result.coords.size() * sizeof(int32_t));
    if (!g_result.feats.empty()) std::memcpy(feats, g_result.feats.data(), g_result.feats.size() * sizeof(float));
}

}  // extern "C"
