// One Pegasos mini-batch step for the L2-regularised hinge loss (paper Sec. 4, "Training":
// mini-batch SGD with Pegasos updates, learning rate 1/(lambda t), each batch half positives and
// half negatives).  The batch is ~B rows of D floats gathered from two resident pools: a few
// megabytes, so the step is bound by launch and memory latency, not bandwidth.
//
//   kernel 1 (margins):  one wave per batch row j: m_j = y_j (<w, x_j> + b);
//                        coef_j = y_j if m_j < 1 else 0           (strict: nothing at the kink)
//   kernel 2 (update):   column d:  w_d <- (1 - eta*lambda) w_d + (eta/B) sum_j coef_j x_{j,d}
//                        each block owns 64 columns, its 16 waves split the batch rows, and the
//                        partial sums are combined in a fixed order (bit-reproducible).
#include "otf_internal.h"

namespace otf {

__device__ __forceinline__ const float *batch_row(int j, const float *Xpos, long long ld_pos, const int32_t *idx_pos,
                                                  int n_pos, const float *Xneg, long long ld_neg,
                                                  const int32_t *idx_neg) {
    return j < n_pos ? Xpos + (long long)idx_pos[j] * ld_pos : Xneg + (long long)idx_neg[j - n_pos] * ld_neg;
}

__global__ __launch_bounds__(256) void sgd_margin_kernel(const float *__restrict__ w, const float *__restrict__ b, int D,
                                                         const float *__restrict__ Xpos, long long ld_pos,
                                                         const int32_t *__restrict__ idx_pos, int n_pos,
                                                         const float *__restrict__ Xneg, long long ld_neg,
                                                         const int32_t *__restrict__ idx_neg, int n_neg,
                                                         float *__restrict__ coef) {
    const int lane = threadIdx.x & 63;
    const int j = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (j >= n_pos + n_neg) return;
    const float *x = batch_row(j, Xpos, ld_pos, idx_pos, n_pos, Xneg, ld_neg, idx_neg);
    float acc = 0.f;
    for (int d = lane * 4; d < D; d += 256) {
        const float4 xv = *reinterpret_cast<const float4 *>(x + d);
        const float4 wv = *reinterpret_cast<const float4 *>(w + d);
        acc = fmaf(xv.x, wv.x, acc);
        acc = fmaf(xv.y, wv.y, acc);
        acc = fmaf(xv.z, wv.z, acc);
        acc = fmaf(xv.w, wv.w, acc);
    }
    acc = wave_sum(acc);
    if (lane == 0) {
        const float y = j < n_pos ? 1.f : -1.f;
        const float margin = y * (acc + (b ? *b : 0.f));
        coef[j] = margin < 1.f ? y : 0.f;
    }
}

__global__ __launch_bounds__(1024) void sgd_update_kernel(float *__restrict__ w, float *__restrict__ b, int D,
                                                          const float *__restrict__ Xpos, long long ld_pos,
                                                          const int32_t *__restrict__ idx_pos, int n_pos,
                                                          const float *__restrict__ Xneg, long long ld_neg,
                                                          const int32_t *__restrict__ idx_neg, int n_neg,
                                                          const float *__restrict__ coef, float shrink, float scale,
                                                          int update_bias) {
    __shared__ float part[16][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int d = blockIdx.x * 64 + lane;
    const int B = n_pos + n_neg;
    // A wave adds its rows j = wave, wave + 16, ... in that order.  The loads of 16 of them are
    // issued together (coefficients, then row numbers, then the values of the violators): taken one
    // row at a time this loop was a chain of dependent memory latencies, 10 us for a batch of 256.
    float acc = 0.f;
    if (d < D) {
        for (int j0 = wave; j0 < B; j0 += 16 * 16) {
            float c[16], xv[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int j = j0 + 16 * i;
                c[i] = j < B ? coef[j] : 0.f;        // same for the whole wave
            }
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                xv[i] = 0.f;
                if (c[i] != 0.f)                     // uniform: only violators are read
                    xv[i] = batch_row(j0 + 16 * i, Xpos, ld_pos, idx_pos, n_pos, Xneg, ld_neg, idx_neg)[d];
            }
#pragma unroll
            for (int i = 0; i < 16; ++i) acc = fmaf(c[i], xv[i], acc);
        }
    }
    part[wave][lane] = acc;
    __syncthreads();
    if (wave == 0 && d < D) {
        float total = 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) total += part[v][lane];
        w[d] = fmaf(shrink, w[d], scale * total);
    }
    if (update_bias && b && blockIdx.x == 0 && threadIdx.x == 0) {
        float ysum = 0.f;
        for (int j = 0; j < B; ++j) ysum += coef[j];
        *b += scale * ysum;
    }
}

hipError_t launch_sgd_step(float *w, float *b, int D, const float *Xpos, int64_t ld_pos, const int32_t *idx_pos,
                           int n_pos, const float *Xneg, int64_t ld_neg, const int32_t *idx_neg, int n_neg,
                           float lambda, int64_t t, int update_bias, float *coef, hipStream_t s) {
    const int B = n_pos + n_neg;
    const double eta = 1.0 / ((double)lambda * (double)t);
    // 1 - eta * lambda = 1 - 1/t whatever lambda is: formed that way it is exactly 0 at t = 1, as the
    // recursion needs (w_1 must not depend on w_0 except through which rows violate)
    const float shrink = (float)(1.0 - 1.0 / (double)t);
    const float scale = (float)(eta / (double)B);
    sgd_margin_kernel<<<(B + 3) / 4, 256, 0, s>>>(w, b, D, Xpos, (long long)ld_pos, idx_pos, n_pos, Xneg,
                                                  (long long)ld_neg, idx_neg, n_neg, coef);
    sgd_update_kernel<<<(D + 63) / 64, 1024, 0, s>>>(w, b, D, Xpos, (long long)ld_pos, idx_pos, n_pos, Xneg,
                                                     (long long)ld_neg, idx_neg, n_neg, coef, shrink, scale,
                                                     update_bias);
    return hipGetLastError();
}

}  // namespace otf
