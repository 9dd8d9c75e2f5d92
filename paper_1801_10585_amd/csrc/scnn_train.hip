// Training-side utilities of the paper that act on a layer's filter: the adaptive density regulariser (Sec. 3.5,
// Eq. 4) and one-warning-shot pruning (Sec. 3.6).  Elementwise over the filter plus one count over the layer's
// output; every sum is formed in a fixed order (integer counts, per-block partial sums added by one thread).
#include "scnn_internal.h"

namespace scnn {

constexpr int kTrainBlocks = 256;  // partial sums per reduction

// two 64-bit counters start at zero (a fill kernel, so that a caller may capture the call in a graph)
__global__ void k_zero_count(unsigned long long* __restrict__ c) {
    if (threadIdx.x < 2 && blockIdx.x == 0) c[threadIdx.x] = 0ull;
}

// Non-zero entries of feats[0 .. rows * channels), rows taken from the device when rows_dev != nullptr.
__global__ __launch_bounds__(256) void k_count_entries(const float* __restrict__ feats, long long rows_imm,
                                                       const long long* __restrict__ rows_dev, long long rows_cap,
                                                       int channels, unsigned long long* __restrict__ count) {
    __shared__ unsigned s_wave[4];
    long long rows = rows_dev ? *rows_dev : rows_imm;
    if (rows > rows_cap) rows = rows_cap;
    const long long n = rows * channels;
    unsigned local = 0;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (long long)gridDim.x * blockDim.x)
        local += feats[i] != 0.0f;
    for (int d = 32; d > 0; d >>= 1) local += __shfl_down(local, d, 64);
    if ((threadIdx.x & 63) == 0) s_wave[threadIdx.x >> 6] = local;
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned t = s_wave[0] + s_wave[1] + s_wave[2] + s_wave[3];
        if (t) atomicAdd(count, (unsigned long long)t);
    }
}

// Eq. 4: the bias of the regulariser from the measured density.
__device__ inline double density_bias(double rho, double rho_up, double o, double b1, double b2) {
    return rho > rho_up ? o + b1 * (rho - rho_up) : -b2 * (rho_up - rho);
}

// grad[i] = 2 * lambda * (w[i] + b) on un-pruned weights (Eq. 3: a pruned weight receives nothing), partial sums of
// lambda * (w[i] + b)^2 per block.
__global__ __launch_bounds__(256) void k_regulariser(const float* __restrict__ w, long long n, double n_total,
                                                     const unsigned long long* __restrict__ count, double rho_up,
                                                     double o, double b1, double b2, double lambda,
                                                     float* __restrict__ grad, double* __restrict__ partial) {
    __shared__ double s_part[256];
    const double rho = (double)*count / n_total;
    const double b = density_bias(rho, rho_up, o, b1, b2);
    double local = 0.0;
    // a block owns one contiguous slice, a thread walks it with stride 256: the order of the additions is fixed
    const long long per = (n + gridDim.x - 1) / gridDim.x;
    const long long lo = (long long)blockIdx.x * per;
    long long hi = lo + per;
    if (hi > n) hi = n;
    for (long long i = lo + threadIdx.x; i < hi; i += 256) {
        const float wi = w[i];
        double g = 0.0;
        if (wi != 0.0f) {
            const double t = (double)wi + b;
            local += t * t;
            g = 2.0 * lambda * t;
        }
        if (grad) grad[i] = (float)g;
    }
    s_part[threadIdx.x] = local;
    __syncthreads();
    if (threadIdx.x == 0) {
        double sum = 0.0;
        for (int i = 0; i < 256; ++i) sum += s_part[i];
        partial[blockIdx.x] = sum;
    }
}

__global__ void k_regulariser_finish(const double* __restrict__ partial, int n_partial,
                                     const unsigned long long* __restrict__ count, double n_total, double rho_up,
                                     double o, double b1, double b2, double lambda, double* __restrict__ out) {
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    double sum = 0.0;
    for (int i = 0; i < n_partial; ++i) sum += partial[i];
    const double rho = (double)*count / n_total;
    out[0] = rho;
    out[1] = density_bias(rho, rho_up, o, b1, b2);
    out[2] = lambda * sum;
    out[3] = (double)*count;
}

hipError_t launch_density_regulariser(const float* feats, long long rows_imm, const long long* rows_dev,
                                      long long rows_cap, int channels, double n_total, double rho_up, double o,
                                      double b1, double b2, double lambda, const float* w, long long n_w, float* grad,
                                      unsigned long long* count, double* partial, double* out, hipStream_t s) {
    hipLaunchKernelGGL(k_zero_count, dim3(1), dim3(64), 0, s, count);
    if (rows_cap > 0) {
        long long blocks = (rows_cap * channels + 255) / 256;
        if (blocks > 2048) blocks = 2048;
        hipLaunchKernelGGL(k_count_entries, dim3((unsigned)blocks), dim3(256), 0, s, feats, rows_imm, rows_dev,
                           rows_cap, channels, count);
    }
    hipLaunchKernelGGL(k_regulariser, dim3(kTrainBlocks), dim3(256), 0, s, w, n_w, n_total, count, rho_up, o, b1, b2,
                       lambda, grad, partial);
    hipLaunchKernelGGL(k_regulariser_finish, dim3(1), dim3(64), 0, s, partial, kTrainBlocks, count, n_total, rho_up, o,
                       b1, b2, lambda, out);
    return hipGetLastError();
}

// One-warning-shot pruning: a weight whose magnitude is below eps at the end of two consecutive epochs is removed
// (set to exactly 0, which the sparse back-propagation then keeps at 0); one that is small for the first time only
// gets its warning.  counts[0] += weights removed by this call, counts[1] = non-zero weights left.
__global__ __launch_bounds__(256) void k_prune(float* __restrict__ w, unsigned char* __restrict__ warned, long long n,
                                               float eps, unsigned long long* __restrict__ counts) {
    __shared__ unsigned s_p[4], s_l[4];
    unsigned pruned = 0, left = 0;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (long long)gridDim.x * blockDim.x) {
        const float wi = w[i];
        const bool small = wi != 0.0f && fabsf(wi) < eps;
        if (small && warned[i]) {
            w[i] = 0.0f;
            warned[i] = 0;
            ++pruned;
        } else {
            warned[i] = small ? 1 : 0;
            left += wi != 0.0f;
        }
    }
    for (int d = 32; d > 0; d >>= 1) {
        pruned += __shfl_down(pruned, d, 64);
        left += __shfl_down(left, d, 64);
    }
    if ((threadIdx.x & 63) == 0) {
        s_p[threadIdx.x >> 6] = pruned;
        s_l[threadIdx.x >> 6] = left;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned p = s_p[0] + s_p[1] + s_p[2] + s_p[3], l = s_l[0] + s_l[1] + s_l[2] + s_l[3];
        if (p) atomicAdd(&counts[0], (unsigned long long)p);
        if (l) atomicAdd(&counts[1], (unsigned long long)l);
    }
}

hipError_t launch_prune(float* w, unsigned char* warned, long long n, float eps, unsigned long long* counts,
                        hipStream_t s) {
    hipLaunchKernelGGL(k_zero_count, dim3(1), dim3(64), 0, s, counts);
    long long blocks = (n + 255) / 256;
    if (blocks < 1) blocks = 1;
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(k_prune, dim3((unsigned)blocks), dim3(256), 0, s, w, warned, n, eps, counts);
    return hipGetLastError();
}

}  // namespace scnn
