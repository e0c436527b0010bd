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
#include <algorithm>

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

// ---------------------------------------------------------------------------------------------
// A whole run of consecutive steps in ONE launch.  (Paper Sec. 4: between two rankings the model
// takes as many steps as fit.  As two launches per step the run is bound by launch and memory
// latency, ~12 us per step; here a step costs one round trip between the workgroups.)
//
// G workgroups of four waves stay resident for the whole run.  Every wave keeps the whole model
// in registers (D <= 2048: 32 values per lane) and the workgroup a master copy in shared memory.
// A step:
//   1. workgroup g owns rows g, g + G, ... of the batch: its waves compute their margins against
//      the model they hold, and add coef_j x_j of their violators to a partial sum vector, from
//      the very registers the row was loaded into (every batch row is read once);
//   2. the waves' vectors are added up through shared memory and the workgroup's partial vector
//      goes to global memory (slot g of this step's parity);
//   3. it announces that (a counter in global memory) and waits until all G have;
//   4. every workgroup adds the G partial vectors, in slot order, into the next model: all hold
//      the same bits, nothing has to be broadcast, and one wait per step suffices (two buffers of
//      partial vectors, by step parity: nobody can be more than one step ahead).
// The wait is BOUNDED: after `spin_limit` polls a workgroup gives up, raises the abort word (the
// others see it in their own polls and stop as well) and the kernel ends; the status word in the
// workspace then reads 1 and the model is unspecified.  All G workgroups must be resident at the
// same time for the waits to end; they need 16 KiB of shared memory and 4 waves each, so they fit
// beside any other kernel of this library, and wait for room otherwise.
constexpr int kPassThreads = 256;
constexpr int kPassMaxG = 32;

struct PassCtl {            // first words of the workspace
    uint32_t status;        // 0 after a complete run, 1 when a wait expired
    uint32_t arrived;       // arrivals so far (G per step)
    uint32_t pad[62];
};
static_assert(sizeof(PassCtl) == 256, "control block");

__global__ void sgd_pass_init_kernel(PassCtl *ctl) {
    ctl->status = 0u;
    ctl->arrived = 0u;
}

template <int NI>   // 256 * NI >= D
__global__ __launch_bounds__(kPassThreads) void sgd_pass_kernel(
    float *__restrict__ w_io, float *__restrict__ b_io, int D, const float *__restrict__ Xpos, long long ld_pos,
    const int32_t *__restrict__ idx_pos, int n_pos, const float *__restrict__ Xneg, long long ld_neg,
    const int32_t *__restrict__ idx_neg, int n_neg, float lambda, long long t_first, int n_steps, int update_bias,
    PassCtl *ctl, float *__restrict__ partial, int DP, uint32_t spin_limit) {
    __shared__ __attribute__((aligned(16))) float wbuf[256 * NI];     // the model (master copy of this workgroup)
    __shared__ __attribute__((aligned(16))) float comb[256 * NI];     // sum of the waves' partial vectors
    __shared__ float s_ysum[4];
    __shared__ uint32_t s_ok;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = blockIdx.x, G = gridDim.x, B = n_pos + n_neg;
    for (int c = tid; c < 256 * NI; c += kPassThreads) wbuf[c] = c < D ? w_io[c] : 0.f;
    float bias = b_io ? *b_io : 0.f;
    __syncthreads();
    float4 wr[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) wr[i] = *reinterpret_cast<const float4 *>(wbuf + 4 * lane + 256 * i);

    bool alive = true;
    for (int s = 0; s < n_steps && alive; ++s) {
        const long long t = t_first + s;
        const double eta = 1.0 / ((double)lambda * (double)t);
        const float shrink = (float)(1.0 - 1.0 / (double)t);
        const float scale = (float)(eta / (double)B);
        const int32_t *ip = idx_pos + (size_t)s * n_pos, *in = idx_neg + (size_t)s * n_neg;
        // 1. margins and partial sums of this wave's rows
        float4 acc[NI];
#pragma unroll
        for (int i = 0; i < NI; ++i) acc[i] = make_float4(0.f, 0.f, 0.f, 0.f);
        float ysum = 0.f;
        // (two rows at a time: the loads of both are in flight before the first is reduced)
        for (int j0 = g + G * wave; j0 < B; j0 += G * 8) {
            const int j1 = j0 + G * 4;
            const bool has1 = j1 < B;                                  // uniform over the wave
            const float *x0 = batch_row(j0, Xpos, ld_pos, ip, n_pos, Xneg, ld_neg, in);
            const float *x1 = has1 ? batch_row(j1, Xpos, ld_pos, ip, n_pos, Xneg, ld_neg, in) : x0;
            float4 xv[2][NI];
#pragma unroll
            for (int i = 0; i < NI; ++i) {
                const int c = 4 * lane + 256 * i;
                const float4 z = make_float4(0.f, 0.f, 0.f, 0.f);
                xv[0][i] = c < D ? *reinterpret_cast<const float4 *>(x0 + c) : z;
                xv[1][i] = c < D ? *reinterpret_cast<const float4 *>(x1 + c) : z;
            }
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                if (h == 1 && !has1) break;
                const int j = h == 0 ? j0 : j1;
                float dot = 0.f;
#pragma unroll
                for (int i = 0; i < NI; ++i) {
                    dot = fmaf(xv[h][i].x, wr[i].x, dot);
                    dot = fmaf(xv[h][i].y, wr[i].y, dot);
                    dot = fmaf(xv[h][i].z, wr[i].z, dot);
                    dot = fmaf(xv[h][i].w, wr[i].w, dot);
                }
                dot = wave_sum(dot);
                const float y = j < n_pos ? 1.f : -1.f;
                const float coef = y * (dot + bias) < 1.f ? y : 0.f;   // strict: nothing at the kink
                if (coef != 0.f) {                                     // uniform over the wave
#pragma unroll
                    for (int i = 0; i < NI; ++i) {
                        acc[i].x = fmaf(coef, xv[h][i].x, acc[i].x);
                        acc[i].y = fmaf(coef, xv[h][i].y, acc[i].y);
                        acc[i].z = fmaf(coef, xv[h][i].z, acc[i].z);
                        acc[i].w = fmaf(coef, xv[h][i].w, acc[i].w);
                    }
                    ysum += coef;
                }
            }
        }
        // 2. the four waves' vectors, added in wave order through shared memory
        for (int v = 0; v < 4; ++v) {
            if (wave == v) {
#pragma unroll
                for (int i = 0; i < NI; ++i) {
                    float4 *p = reinterpret_cast<float4 *>(comb + 4 * lane + 256 * i);
                    float4 a = acc[i];
                    if (v > 0) {
                        const float4 o = *p;
                        a = make_float4(o.x + a.x, o.y + a.y, o.z + a.z, o.w + a.w);
                    }
                    *p = a;
                }
                if (lane == 0) s_ysum[v] = ysum;
            }
            __syncthreads();
        }
        float *mine = partial + ((size_t)(s & 1) * G + g) * DP;
        for (int c = tid * 4; c < D; c += kPassThreads * 4)
            *reinterpret_cast<float4 *>(mine + c) = *reinterpret_cast<const float4 *>(comb + c);
        if (tid == 0) mine[D] = (s_ysum[0] + s_ysum[1]) + (s_ysum[2] + s_ysum[3]);
        // 3. announce, and wait for the others (bounded)
        __syncthreads();                                               // the workgroup's stores have been issued and waited for
        if (tid == 0) {
            __hip_atomic_fetch_add(&ctl->arrived, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
            const uint32_t target = (uint32_t)G * (uint32_t)(s + 1);
            uint32_t ok = 0u;
            for (uint32_t it = 0; it < spin_limit; ++it) {
                if (__hip_atomic_load(&ctl->arrived, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= target) {
                    ok = 1u;
                    break;
                }
                // (the abort word is looked at every 64th poll: a poll is a round trip to memory)
                if ((it & 63u) == 63u && __hip_atomic_load(&ctl->status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) break;
            }
            if (!ok) __hip_atomic_store(&ctl->status, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");         // the others' partial vectors, not stale cache lines
            s_ok = ok;
        }
        __syncthreads();
        alive = s_ok != 0u;                                            // uniform over the workgroup
        if (!alive) break;
        // 4. the next model, from all partial vectors in slot order (the same bits in every workgroup)
        const float *all = partial + (size_t)(s & 1) * G * DP;
        for (int c = tid * 4; c < D; c += kPassThreads * 4) {
            float4 tot = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll 1
            for (int h0 = 0; h0 < G; h0 += 32) {                        // 32 loads in flight together
                float4 p[32];
#pragma unroll
                for (int h = 0; h < 32; ++h)
                    p[h] = *reinterpret_cast<const float4 *>(all + (size_t)(h0 + h < G ? h0 + h : 0) * DP + c);
#pragma unroll
                for (int h = 0; h < 32; ++h)
                    if (h0 + h < G) tot = make_float4(tot.x + p[h].x, tot.y + p[h].y, tot.z + p[h].z, tot.w + p[h].w);
            }
            float4 wv = *reinterpret_cast<const float4 *>(wbuf + c);
            wv.x = fmaf(shrink, wv.x, scale * tot.x);
            wv.y = fmaf(shrink, wv.y, scale * tot.y);
            wv.z = fmaf(shrink, wv.z, scale * tot.z);
            wv.w = fmaf(shrink, wv.w, scale * tot.w);
            *reinterpret_cast<float4 *>(wbuf + c) = wv;
        }
        if (update_bias && b_io) {
            float ys = 0.f;
            for (int h = 0; h < G; ++h) ys += all[(size_t)h * DP + D];
            bias += scale * ys;
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < NI; ++i) wr[i] = *reinterpret_cast<const float4 *>(wbuf + 4 * lane + 256 * i);
    }
    if (g == 0 && alive) {
        for (int c = tid; c < D; c += kPassThreads) w_io[c] = wbuf[c];
        if (update_bias && b_io && tid == 0) *b_io = bias;
    }
}

hipError_t launch_sgd_pass_clear_status(void *ws, hipStream_t s) {
    sgd_pass_init_kernel<<<1, 1, 0, s>>>(reinterpret_cast<PassCtl *>(ws));
    return hipGetLastError();
}

size_t sgd_pass_ws_bytes(int D) {
    const int DP = (D + 4 + 63) / 64 * 64;
    return sizeof(PassCtl) + (size_t)2 * kPassMaxG * DP * sizeof(float);
}

// True when the one-launch run applies (the model fits the waves' registers).
bool sgd_pass_fits(int D) { return D <= 2048; }

hipError_t launch_sgd_pass(float *w, float *b, int D, const float *Xpos, int64_t ld_pos, const int32_t *idx_pos,
                           int n_pos, const float *Xneg, int64_t ld_neg, const int32_t *idx_neg, int n_neg,
                           float lambda, int64_t t_first, int n_steps, int update_bias, void *ws, uint32_t spin_limit,
                           hipStream_t s) {
    const int B = n_pos + n_neg;
    const int DP = (D + 4 + 63) / 64 * 64;
    PassCtl *ctl = reinterpret_cast<PassCtl *>(ws);
    float *partial = reinterpret_cast<float *>(reinterpret_cast<uint8_t *>(ws) + sizeof(PassCtl));
    const int G = B < kPassMaxG ? B : kPassMaxG;
    sgd_pass_init_kernel<<<1, 1, 0, s>>>(ctl);
#define OTF_PASS(NI)                                                                                                  \
    sgd_pass_kernel<NI><<<G, kPassThreads, 0, s>>>(w, b, D, Xpos, (long long)ld_pos, idx_pos, n_pos, Xneg,             \
                                                   (long long)ld_neg, idx_neg, n_neg, lambda, (long long)t_first,      \
                                                   n_steps, update_bias, ctl, partial, DP, spin_limit)
    if (D <= 256) OTF_PASS(1);
    else if (D <= 512) OTF_PASS(2);
    else if (D <= 1024) OTF_PASS(4);
    else OTF_PASS(8);
#undef OTF_PASS
    return hipGetLastError();
}

// Counts the entries of idx[0..n) outside [0, rows): a pool's row numbers are read unchecked by the
// training kernels (they carry no pool sizes), so a caller checks them once when it builds them.
__global__ __launch_bounds__(256) void check_indices_kernel(const int32_t *__restrict__ idx, long long n, long long rows,
                                                            int32_t *bad) {
    int mine = 0;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (long long)gridDim.x * blockDim.x)
        mine += (idx[i] < 0 || (long long)idx[i] >= rows) ? 1 : 0;
    if (mine) atomicAdd(bad, mine);
}

hipError_t launch_check_indices(const int32_t *idx, int64_t n, int64_t rows, int32_t *bad, hipStream_t s) {
    const int blocks = (int)std::min<int64_t>((n + 255) / 256, 1024);
    check_indices_kernel<<<blocks < 1 ? 1 : blocks, 256, 0, s>>>(idx, (long long)n, (long long)rows, bad);
    return hipGetLastError();
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
