// Batch norm (training mode, statistics of the worker's own shard) and the
// bias / ReLU backward, all as per-channel column reductions over a row-major
// [M][C] activation matrix followed by an elementwise pass.  HBM-bound.
//
// Reduction scheme (deterministic, no atomics): the rows are cut into at most
// kRedRowBlocks blocks; a workgroup of TX x TY lanes owns 32*VEC channels of
// one row block, each lane accumulating one 16-byte channel vector over every
// TY-th row in float32; lanes are combined through LDS; a second tiny kernel
// adds the row blocks in float64.
#include <type_traits>

#include "dev_common.h"
#include "kernels.h"
#include "profiler.h"
#include "tune.h"

namespace edl {

constexpr float kBnEps = 1e-5f;
constexpr float kBnRunningMomentum = 0.1f;

struct RedShape {
    int TX, TY, cvecs, row_blocks, rows_per_block;
    dim3 grid, block;
};

static RedShape red_shape(int64_t M, int C, int VEC) {
    RedShape s;
    s.cvecs = (C + VEC - 1) / VEC;
    int tx = 1;
    while (tx < s.cvecs && tx < 32) tx <<= 1;
    s.TX = tx;
    s.TY = 256 / tx;
    const int col_blocks = (s.cvecs + tx - 1) / tx;
    // aim at ~2048 workgroups, at least TY*4 rows each
    int64_t rb = (2048 + col_blocks - 1) / col_blocks;
    const int64_t max_rb = (M + (int64_t)s.TY * 4 - 1) / ((int64_t)s.TY * 4);
    if (rb > max_rb) rb = max_rb;
    if (rb > kRedRowBlocks) rb = kRedRowBlocks;
    if (rb < 1) rb = 1;
    s.rows_per_block = (int)((M + rb - 1) / rb);
    s.row_blocks = (int)((M + s.rows_per_block - 1) / s.rows_per_block);
    s.grid = dim3(col_blocks, s.row_blocks);
    s.block = dim3(s.TX, s.TY);
    return s;
}

// Loads VEC channels of row r starting at channel c0 (zero beyond C).
template <typename T, int VEC>
__device__ __forceinline__ void load_row(const T* base, int64_t r, int C, int c0, float (&out)[VEC]) {
    if (VEC > 1) {
        const Vec16<T> v = load_vec(base + r * C + c0);
        #pragma unroll
        for (int e = 0; e < VEC; ++e) out[e] = Elem<T>::to_f32(v.e[e]);
    } else {
        out[0] = Elem<T>::to_f32(base[r * C + c0]);
    }
}

// the same through a non-temporal load: for a tensor this pass reads once and nothing reads again soon
typedef unsigned int nt_u32x4 __attribute__((ext_vector_type(4)));
template <typename T, int VEC>
__device__ __forceinline__ void load_row_nt(const T* base, int64_t r, int C, int c0, float (&out)[VEC]) {
    if (VEC > 1) {
        Vec16<T> v;
        const nt_u32x4 q = __builtin_nontemporal_load(reinterpret_cast<const nt_u32x4*>(base + r * C + c0));
        v.u = make_uint4(q.x, q.y, q.z, q.w);
        #pragma unroll
        for (int e = 0; e < VEC; ++e) out[e] = Elem<T>::to_f32(v.e[e]);
    } else {
        out[0] = Elem<T>::to_f32(base[r * C + c0]);
    }
}

template <typename T, int VEC>
__device__ __forceinline__ void store_row(T* base, int64_t r, int C, int c0, const float (&in)[VEC]) {
    if (VEC > 1) {
        Vec16<T> v;
        #pragma unroll
        for (int e = 0; e < VEC; ++e) v.e[e] = Elem<T>::from_f32(in[e]);
        store_vec(base + r * C + c0, v);
    } else {
        base[r * C + c0] = Elem<T>::from_f32(in[0]);
    }
}

// KIND 0: a = x, b = x^2                       (batch-norm statistics)
// KIND 1: a = dy', b = dy' * xhat              (batch-norm backward sums), dy' = dy * (y>0) if relu
// KIND 2: a = dy' (written back in place), b=0 (bias gradient / ReLU mask)
template <typename T, int VEC, int KIND>
__global__ __launch_bounds__(256) void colreduce_kernel(const T* __restrict__ x, const T* __restrict__ y, T* dy,
                                                        const float* __restrict__ mean_rstd, int64_t M, int C,
                                                        int rows_per_block, int relu, float* __restrict__ partial) {
    __shared__ float red[2][256 * VEC];
    const int tx = threadIdx.x, ty = threadIdx.y, TX = blockDim.x, TY = blockDim.y;
    const int c0 = (blockIdx.x * TX + tx) * VEC;
    const bool active = c0 < C;
    float a[VEC], b[VEC];
    #pragma unroll
    for (int e = 0; e < VEC; ++e) { a[e] = 0.f; b[e] = 0.f; }
    float mu[VEC], rs[VEC];
    if (KIND == 1 && active) {
        #pragma unroll
        for (int e = 0; e < VEC; ++e) { mu[e] = mean_rstd[c0 + e]; rs[e] = mean_rstd[C + c0 + e]; }
    }
    const int64_t r0 = (int64_t)blockIdx.y * rows_per_block;
    int64_t r1 = r0 + rows_per_block;
    if (r1 > M) r1 = M;
    if (active) {
        // U rows per trip, every load of a trip issued before the first use: the loads are unconditional
        // (without ReLU y is a valid tensor that is read and ignored), so none of them waits for another.
        auto rows = [&](int64_t r, auto ucount) {
            constexpr int U = decltype(ucount)::value;
            float xv[U][VEC], yv[U][VEC], g[U][VEC];
            #pragma unroll
            for (int u = 0; u < U; ++u) {
                const int64_t rr = r + (int64_t)u * TY;
                if (KIND == 0) {
                    load_row<T, VEC>(x, rr, C, c0, xv[u]);
                } else {
                    load_row<T, VEC>(dy, rr, C, c0, g[u]);
                    load_row<T, VEC>(y, rr, C, c0, yv[u]);
                    if (KIND == 1) load_row<T, VEC>(x, rr, C, c0, xv[u]);
                }
            }
            #pragma unroll
            for (int u = 0; u < U; ++u) {
                if (KIND == 0) {
                    #pragma unroll
                    for (int e = 0; e < VEC; ++e) { a[e] += xv[u][e]; b[e] += xv[u][e] * xv[u][e]; }
                } else {
                    #pragma unroll
                    for (int e = 0; e < VEC; ++e) g[u][e] = (!relu || yv[u][e] > 0.f) ? g[u][e] : 0.f;
                    if (KIND == 1) {
                        #pragma unroll
                        for (int e = 0; e < VEC; ++e) { a[e] += g[u][e]; b[e] += g[u][e] * ((xv[u][e] - mu[e]) * rs[e]); }
                    } else {
                        if (relu) store_row<T, VEC>(dy, r + (int64_t)u * TY, C, c0, g[u]);
                        #pragma unroll
                        for (int e = 0; e < VEC; ++e) a[e] += g[u][e];
                    }
                }
            }
        };
        int64_t r = r0 + ty;
        for (; r + TY < r1; r += 2 * (int64_t)TY) rows(r, std::integral_constant<int, 2>());
        if (r < r1) rows(r, std::integral_constant<int, 1>());
    }
    const int lane = ty * TX + tx;
    #pragma unroll
    for (int e = 0; e < VEC; ++e) { red[0][lane * VEC + e] = a[e]; red[1][lane * VEC + e] = b[e]; }
    __syncthreads();
    if (ty == 0 && active) {
        for (int j = 1; j < TY; ++j) {
            #pragma unroll
            for (int e = 0; e < VEC; ++e) {
                a[e] += red[0][(j * TX + tx) * VEC + e];
                b[e] += red[1][(j * TX + tx) * VEC + e];
            }
        }
        // partial[sum kind][channel][row block]: a channel's partial sums are contiguous for the finishing kernel
        #pragma unroll
        for (int e = 0; e < VEC; ++e) {
            if (c0 + e < C) {
                partial[(int64_t)(c0 + e) * kRedRowBlocks + blockIdx.y] = a[e];
                partial[(int64_t)(C + c0 + e) * kRedRowBlocks + blockIdx.y] = b[e];
            }
        }
    }
}

// Sum of the row blocks' partial sums of one channel: one wave per channel, lane
// L takes blocks L, L+64, ... (coalesced) in float64, then a butterfly.
// blockDim = 256 = 4 channels x 64 lanes.
__device__ __forceinline__ void sum_partials(const float* __restrict__ partial, int row_blocks, int C, int c, int sub,
                                             double& s, double& q) {
    s = 0;
    q = 0;
    if (c < C) {
        const float* ps = partial + (int64_t)c * kRedRowBlocks;
        const float* pq = partial + (int64_t)(C + c) * kRedRowBlocks;
        // four loads of each kind in flight per lane (the partial sums of a channel are contiguous)
        int j = sub;
        for (; j + 192 < row_blocks; j += 256) {
            const float s0 = ps[j], s1 = ps[j + 64], s2 = ps[j + 128], s3 = ps[j + 192];
            const float q0 = pq[j], q1 = pq[j + 64], q2 = pq[j + 128], q3 = pq[j + 192];
            s += (double)s0; s += (double)s1; s += (double)s2; s += (double)s3;
            q += (double)q0; q += (double)q1; q += (double)q2; q += (double)q3;
        }
        for (; j < row_blocks; j += 64) {
            s += (double)ps[j];
            q += (double)pq[j];
        }
    }
    for (int o = 32; o > 0; o >>= 1) {
        s += __shfl_xor(s, o, 64);
        q += __shfl_xor(q, o, 64);
    }
}

// mean / rstd from the partial sums; running statistics of the worker whose
// model a joiner would receive (unbiased variance, momentum 0.1)
__global__ __launch_bounds__(256) void bn_stats_finalize_kernel(const float* __restrict__ partial, int row_blocks, int64_t M,
                                                                int C, float* __restrict__ mean_rstd, float* running) {
    const int c = blockIdx.x * 4 + (threadIdx.x >> 6), sub = threadIdx.x & 63;
    double s, q;
    sum_partials(partial, row_blocks, C, c, sub, s, q);
    if (c >= C || sub != 0) return;
    const double mean = s / (double)M;
    double var = q / (double)M - mean * mean;
    if (var < 0) var = 0;
    mean_rstd[c] = (float)mean;
    mean_rstd[C + c] = (float)(1.0 / sqrt(var + (double)kBnEps));
    if (running) {
        const double unbiased = M > 1 ? var * (double)M / (double)(M - 1) : var;
        running[c] = (1.f - kBnRunningMomentum) * running[c] + kBnRunningMomentum * (float)mean;
        running[C + c] = (1.f - kBnRunningMomentum) * running[C + c] + kBnRunningMomentum * (float)unbiased;
    }
}

// dgamma = sum dy'*xhat, dbeta = sum dy'; coef = {dbeta/M, dgamma/M}
__global__ __launch_bounds__(256) void bn_bwd_finalize_kernel(const float* __restrict__ partial, int row_blocks, int64_t M,
                                                              int C, float* __restrict__ dgamma, float* __restrict__ dbeta,
                                                              float* __restrict__ coef) {
    const int c = blockIdx.x * 4 + (threadIdx.x >> 6), sub = threadIdx.x & 63;
    double s, q;
    sum_partials(partial, row_blocks, C, c, sub, s, q);
    if (c >= C || sub != 0) return;
    dbeta[c] = (float)s;
    dgamma[c] = (float)q;
    coef[c] = (float)(s / (double)M);
    coef[C + c] = (float)(q / (double)M);
}

__global__ __launch_bounds__(256) void bias_finalize_kernel(const float* __restrict__ partial, int row_blocks, int C,
                                                            float* __restrict__ dbias) {
    const int c = blockIdx.x * 4 + (threadIdx.x >> 6), sub = threadIdx.x & 63;
    double s, q;
    sum_partials(partial, row_blocks, C, c, sub, s, q);
    if (c >= C || sub != 0) return;
    dbias[c] = (float)s;
}

// y = relu(gamma * (x - mean) * rstd + beta + res)
// No load sits behind a run-time branch, so that all of a lane's loads are in flight together.
template <typename T, int VEC, bool RES, bool NT>
__global__ __launch_bounds__(256) void bn_apply_kernel(const T* __restrict__ x, const T* __restrict__ res,
                                                       T* __restrict__ y, const float* __restrict__ gamma,
                                                       const float* __restrict__ beta, const float* __restrict__ mean_rstd,
                                                       int64_t M, int C, int cvecs, int relu) {
    const int64_t total = M * cvecs;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
        const int64_t r = i / cvecs;
        const int c0 = (int)(i - r * cvecs) * VEC;
        float xv[VEC], rv[VEC], out[VEC];
        if (NT) load_row_nt<T, VEC>(x, r, C, c0, xv); else load_row<T, VEC>(x, r, C, c0, xv);
        if (RES) { if (NT) load_row_nt<T, VEC>(res, r, C, c0, rv); else load_row<T, VEC>(res, r, C, c0, rv); }
        #pragma unroll
        for (int e = 0; e < VEC; ++e) {
            const float sc = gamma[c0 + e] * mean_rstd[C + c0 + e];
            out[e] = (xv[e] - mean_rstd[c0 + e]) * sc + beta[c0 + e];
            if (RES) out[e] += rv[e];
            if (relu) out[e] = out[e] > 0.f ? out[e] : 0.f;
        }
        store_row<T, VEC>(y, r, C, c0, out);
    }
}

// dx = gamma*rstd*(dy' - coef0 - xhat*coef1) ; dres (+)= dy'
// MASK: dy' = dy * (y > 0) is formed here (else dy arrives masked, or there is no ReLU, and y is not read);
// ACC: dres already holds a gradient that dy' is added to.  Compile-time, so that no load sits behind a
// run-time branch and none is issued that is not needed.
template <typename T, int VEC, bool MASK, bool ACC, bool NT>
__global__ __launch_bounds__(256) void bn_bwd_apply_kernel(const T* __restrict__ x, const T* __restrict__ y,
                                                           const T* __restrict__ dy, T* __restrict__ dx, T* dres,
                                                           const float* __restrict__ gamma,
                                                           const float* __restrict__ mean_rstd,
                                                           const float* __restrict__ coef, int64_t M, int C, int cvecs) {
    const int64_t total = M * cvecs;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
        const int64_t r = i / cvecs;
        const int c0 = (int)(i - r * cvecs) * VEC;
        float xv[VEC], yv[VEC], g[VEC], old[VEC], out[VEC];
        if (NT) load_row_nt<T, VEC>(x, r, C, c0, xv); else load_row<T, VEC>(x, r, C, c0, xv);
        load_row<T, VEC>(dy, r, C, c0, g);
        if (MASK) { if (NT) load_row_nt<T, VEC>(y, r, C, c0, yv); else load_row<T, VEC>(y, r, C, c0, yv); }
        if (ACC) load_row<T, VEC>(dres, r, C, c0, old);
        #pragma unroll
        for (int e = 0; e < VEC; ++e) {
            if (MASK) g[e] = yv[e] > 0.f ? g[e] : 0.f;
            const float rs = mean_rstd[C + c0 + e];
            const float xh = (xv[e] - mean_rstd[c0 + e]) * rs;
            out[e] = gamma[c0 + e] * rs * (g[e] - coef[c0 + e] - xh * coef[C + c0 + e]);
        }
        store_row<T, VEC>(dx, r, C, c0, out);
        if (dres) {
            if (ACC) {
                #pragma unroll
                for (int e = 0; e < VEC; ++e) g[e] += old[e];
            }
            store_row<T, VEC>(dres, r, C, c0, g);
        }
    }
}

static inline int ew_grid(int64_t total) {
    int64_t b = (total + 255) / 256;
    if (b > (1 << 30)) b = 1 << 30;
    if (b < 1) b = 1;
    return (int)b;
}

template <typename T, int VEC>
static void bn_forward_t(const void* x, const void* res, void* y, const float* gamma, const float* beta,
                         float* save, float* running, int64_t M, int C, bool relu, float* partial, int stats_row_blocks,
                         hipStream_t st) {
    const RedShape s = red_shape(M, C, VEC);
    const double tb = (double)sizeof(T) * (double)M * C;   // bytes of one [M][C] tensor
    if (stats_row_blocks <= 0) {   // else the producer of x left the partial sums
        ProfScope ps(prof_shape_label("bn_stats", M, C), 0.0, tb, st);
        hipLaunchKernelGGL((colreduce_kernel<T, VEC, 0>), s.grid, s.block, 0, st, (const T*)x, (const T*)nullptr, (T*)nullptr,
                           (const float*)nullptr, M, C, s.rows_per_block, 0, partial);
        stats_row_blocks = s.row_blocks;
    }
    {
        ProfScope ps("bn_stats_finalize", 0.0, 8.0 * (double)stats_row_blocks * C, st);
        hipLaunchKernelGGL(bn_stats_finalize_kernel, dim3((C + 3) / 4), dim3(256), 0, st, partial, stats_row_blocks, M, C,
                           save, running);
    }
    ProfScope ps(prof_shape_label("bn_apply", M, C), 0.0, tb * (res ? 3.0 : 2.0), st);
    const bool nt = tune().bn_nt != 0 && tb >= (double)tune().bn_nt_bytes;
#define EDL_BN_APPLY(RES, NT)                                                                                          \
    hipLaunchKernelGGL((bn_apply_kernel<T, VEC, RES, NT>), dim3(ew_grid(M * s.cvecs)), dim3(256), 0, st, (const T*)x, \
                       (const T*)res, (T*)y, gamma, beta, save, M, C, s.cvecs, relu ? 1 : 0)
    if (res) { if (nt) EDL_BN_APPLY(true, true); else EDL_BN_APPLY(true, false); }
    else { if (nt) EDL_BN_APPLY(false, true); else EDL_BN_APPLY(false, false); }
#undef EDL_BN_APPLY
}

void launch_bn_forward(int dtype, const void* x, const void* res, void* y, const float* gamma, const float* beta,
                       float* save, float* running, int64_t M, int C, bool relu, float* partial, int stats_row_blocks,
                       hipStream_t st) {
    if (dtype == 1) {
        if (C % 8 == 0) bn_forward_t<bf16_t, 8>(x, res, y, gamma, beta, save, running, M, C, relu, partial, stats_row_blocks, st);
        else bn_forward_t<bf16_t, 1>(x, res, y, gamma, beta, save, running, M, C, relu, partial, stats_row_blocks, st);
    } else {
        if (C % 4 == 0) bn_forward_t<float, 4>(x, res, y, gamma, beta, save, running, M, C, relu, partial, stats_row_blocks, st);
        else bn_forward_t<float, 1>(x, res, y, gamma, beta, save, running, M, C, relu, partial, stats_row_blocks, st);
    }
}

template <typename T, int VEC>
static void bn_backward_t(const void* x, const void* y, const void* dy, void* dx, void* dres, bool dres_acc,
                          const float* gamma, const float* save, float* dgamma, float* dbeta, int64_t M, int C,
                          bool relu, float* partial, float* coef, int sums_row_blocks, hipStream_t st) {
    const RedShape s = red_shape(M, C, VEC);
    const double tb = (double)sizeof(T) * (double)M * C;
    const bool fused = sums_row_blocks > 0;
    if (sums_row_blocks <= 0) {   // else the dgrad that produced dy left the sums
        ProfScope ps(prof_shape_label("bn_bwd_reduce", M, C), 0.0, tb * (relu ? 3.0 : 2.0), st);
        hipLaunchKernelGGL((colreduce_kernel<T, VEC, 1>), s.grid, s.block, 0, st, (const T*)x, (const T*)(relu ? y : x), (T*)dy, save,
                           M, C, s.rows_per_block, relu ? 1 : 0, partial);
        sums_row_blocks = s.row_blocks;
    }
    {
        ProfScope ps("bn_bwd_finalize", 0.0, 8.0 * (double)sums_row_blocks * C, st);
        hipLaunchKernelGGL(bn_bwd_finalize_kernel, dim3((C + 3) / 4), dim3(256), 0, st, partial, sums_row_blocks, M, C,
                           dgamma, dbeta, coef);
    }
    // the dgrad that left the sums also left dy masked: the activation is then not read again
    const bool mask = relu && !fused;
    const bool acc = dres && dres_acc;
    ProfScope ps(prof_shape_label("bn_bwd_apply", M, C), 0.0, tb * ((mask ? 3.0 : 2.0) + 1.0 + (dres ? (acc ? 2.0 : 1.0) : 0.0)), st);
    const dim3 grid(ew_grid(M * s.cvecs));
    const bool nt = tune().bn_nt != 0 && tb >= (double)tune().bn_nt_bytes;
#define EDL_BN_BWD_APPLY(MASK, ACC)                                                                                       \
    do {                                                                                                                  \
        if (nt) hipLaunchKernelGGL((bn_bwd_apply_kernel<T, VEC, MASK, ACC, true>), grid, dim3(256), 0, st, (const T*)x, (const T*)y, (const T*)dy, \
                                   (T*)dx, (T*)dres, gamma, save, coef, M, C, s.cvecs);                                  \
        else hipLaunchKernelGGL((bn_bwd_apply_kernel<T, VEC, MASK, ACC, false>), grid, dim3(256), 0, st, (const T*)x, (const T*)y, (const T*)dy, \
                                (T*)dx, (T*)dres, gamma, save, coef, M, C, s.cvecs);                                     \
    } while (0)
    if (mask) { if (acc) EDL_BN_BWD_APPLY(true, true); else EDL_BN_BWD_APPLY(true, false); }
    else { if (acc) EDL_BN_BWD_APPLY(false, true); else EDL_BN_BWD_APPLY(false, false); }
#undef EDL_BN_BWD_APPLY
}

void launch_bn_backward(int dtype, const void* x, const void* y, const void* dy, void* dx, void* dres,
                        bool dres_accumulate, const float* gamma, const float* save, float* dgamma, float* dbeta,
                        int64_t M, int C, bool relu, float* partial, float* coef, int sums_row_blocks,
                        hipStream_t st) {
    if (dtype == 1) {
        if (C % 8 == 0) bn_backward_t<bf16_t, 8>(x, y, dy, dx, dres, dres_accumulate, gamma, save, dgamma, dbeta, M, C, relu, partial, coef, sums_row_blocks, st);
        else bn_backward_t<bf16_t, 1>(x, y, dy, dx, dres, dres_accumulate, gamma, save, dgamma, dbeta, M, C, relu, partial, coef, sums_row_blocks, st);
    } else {
        if (C % 4 == 0) bn_backward_t<float, 4>(x, y, dy, dx, dres, dres_accumulate, gamma, save, dgamma, dbeta, M, C, relu, partial, coef, sums_row_blocks, st);
        else bn_backward_t<float, 1>(x, y, dy, dx, dres, dres_accumulate, gamma, save, dgamma, dbeta, M, C, relu, partial, coef, sums_row_blocks, st);
    }
}

template <typename T, int VEC>
static void bias_relu_backward_t(const void* y, void* dy, float* dbias, int64_t M, int C, bool relu, float* partial,
                                 int sums_row_blocks, hipStream_t st) {
    const RedShape s = red_shape(M, C, VEC);
    const double tb = (double)sizeof(T) * (double)M * C;
    if (sums_row_blocks <= 0) {   // else dy is masked already and its column sums are in partial
        ProfScope ps("bias_relu_bwd", 0.0, tb * (relu ? 3.0 : 1.0), st);
        hipLaunchKernelGGL((colreduce_kernel<T, VEC, 2>), s.grid, s.block, 0, st, (const T*)nullptr, (const T*)(relu ? y : dy), (T*)dy,
                           (const float*)nullptr, M, C, s.rows_per_block, relu ? 1 : 0, partial);
        sums_row_blocks = s.row_blocks;
    }
    if (dbias) {
        ProfScope ps("bias_finalize", 0.0, 4.0 * (double)sums_row_blocks * C, st);
        hipLaunchKernelGGL(bias_finalize_kernel, dim3((C + 3) / 4), dim3(256), 0, st, partial, sums_row_blocks, C, dbias);
    }
}

void launch_bias_relu_backward(int dtype, const void* y, void* dy, float* dbias, int64_t M, int C, bool relu,
                               float* partial, int sums_row_blocks, hipStream_t st) {
    if (!relu && !dbias) return;
    if (dtype == 1) {
        if (C % 8 == 0) bias_relu_backward_t<bf16_t, 8>(y, dy, dbias, M, C, relu, partial, sums_row_blocks, st);
        else bias_relu_backward_t<bf16_t, 1>(y, dy, dbias, M, C, relu, partial, sums_row_blocks, st);
    } else {
        if (C % 4 == 0) bias_relu_backward_t<float, 4>(y, dy, dbias, M, C, relu, partial, sums_row_blocks, st);
        else bias_relu_backward_t<float, 1>(y, dy, dbias, M, C, relu, partial, sums_row_blocks, st);
    }
}

}  // namespace edl
