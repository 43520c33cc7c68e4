// Pooling and the softmax cross-entropy loss.  All HBM- or latency-bound.
#include "dev_common.h"
#include "kernels.h"
#include "profiler.h"

namespace edl {

static inline int ew_grid(int64_t total) {
    int64_t b = (total + 255) / 256;
    if (b > (1 << 30)) b = 1 << 30;
    if (b < 1) b = 1;
    return (int)b;
}

// ---------------------------------------------------------------------------
// max pool: one lane per output element (channel innermost, so neighbouring
// lanes read neighbouring channels).  arg = r*k + s of the first maximum in
// row-major window order (255 = no tap in range, which cannot happen for the
// geometries used).
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void maxpool_fwd_kernel(const T* __restrict__ x, T* __restrict__ y,
                                                          uint8_t* __restrict__ arg, int N, int H, int W, int C, int k,
                                                          int stride, int pad, int Ho, int Wo) {
    const int64_t total = (int64_t)N * Ho * Wo * C;
    const int64_t step = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += step) {
        const int c = (int)(i % C);
        int64_t t = i / C;
        const int wo = (int)(t % Wo); t /= Wo;
        const int ho = (int)(t % Ho);
        const int n = (int)(t / Ho);
        float best = 0.f;
        int where = 255;
        for (int r = 0; r < k; ++r) {
            const int h = ho * stride - pad + r;
            if (h < 0 || h >= H) continue;
            for (int s = 0; s < k; ++s) {
                const int w = wo * stride - pad + s;
                if (w < 0 || w >= W) continue;
                const float v = Elem<T>::to_f32(x[(((int64_t)n * H + h) * W + w) * C + c]);
                if (where == 255 || v > best) { best = v; where = r * k + s; }
            }
        }
        y[i] = Elem<T>::from_f32(best);
        arg[i] = (uint8_t)where;
    }
}

// gather form of the backward: an input element collects dy from every window
// that recorded it as its arg-max (no atomics, deterministic)
template <typename T>
__global__ __launch_bounds__(256) void maxpool_bwd_kernel(const T* __restrict__ dy, const uint8_t* __restrict__ arg,
                                                          T* dx, int accumulate, int N, int H, int W, int C, int k,
                                                          int stride, int pad, int Ho, int Wo) {
    const int64_t total = (int64_t)N * H * W * C;
    const int64_t step = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += step) {
        const int c = (int)(i % C);
        int64_t t = i / C;
        const int w = (int)(t % W); t /= W;
        const int h = (int)(t % H);
        const int n = (int)(t / H);
        float g = 0.f;
        for (int r = 0; r < k; ++r) {
            const int hn = h + pad - r;
            if (hn < 0 || hn % stride) continue;
            const int ho = hn / stride;
            if (ho >= Ho) continue;
            for (int s = 0; s < k; ++s) {
                const int wn = w + pad - s;
                if (wn < 0 || wn % stride) continue;
                const int wo = wn / stride;
                if (wo >= Wo) continue;
                const int64_t o = (((int64_t)n * Ho + ho) * Wo + wo) * C + c;
                if (arg[o] == r * k + s) g += Elem<T>::to_f32(dy[o]);
            }
        }
        if (accumulate) g += Elem<T>::to_f32(dx[i]);
        dx[i] = Elem<T>::from_f32(g);
    }
}

// 16-byte channel vectors per lane (C a multiple of the vector width)
template <typename T>
__global__ __launch_bounds__(256) void maxpool_fwd_vec_kernel(const T* __restrict__ x, T* __restrict__ y,
                                                              uint8_t* __restrict__ arg, int N, int H, int W, int C, int k,
                                                              int stride, int pad, int Ho, int Wo) {
    constexpr int VEC = Elem<T>::VEC;
    const int cv = C / VEC;
    const int64_t total = (int64_t)N * Ho * Wo * cv;
    const int64_t step = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += step) {
        const int c0 = (int)(i % cv) * VEC;
        int64_t t = i / cv;
        const int wo = (int)(t % Wo); t /= Wo;
        const int ho = (int)(t % Ho);
        const int n = (int)(t / Ho);
        float best[VEC];
        int where[VEC];
        #pragma unroll
        for (int e = 0; e < VEC; ++e) { best[e] = 0.f; where[e] = 255; }
        for (int r = 0; r < k; ++r) {
            const int h = ho * stride - pad + r;
            if (h < 0 || h >= H) continue;
            for (int s = 0; s < k; ++s) {
                const int w = wo * stride - pad + s;
                if (w < 0 || w >= W) continue;
                const Vec16<T> v = load_vec(x + (((int64_t)n * H + h) * W + w) * C + c0);
                #pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    const float f = Elem<T>::to_f32(v.e[e]);
                    if (where[e] == 255 || f > best[e]) { best[e] = f; where[e] = r * k + s; }
                }
            }
        }
        const int64_t o = ((((int64_t)n * Ho + ho) * Wo + wo) * C) + c0;
        Vec16<T> out;
        #pragma unroll
        for (int e = 0; e < VEC; ++e) { out.e[e] = Elem<T>::from_f32(best[e]); arg[o + e] = (uint8_t)where[e]; }
        store_vec(y + o, out);
    }
}

template <typename T>
__global__ __launch_bounds__(256) void maxpool_bwd_vec_kernel(const T* __restrict__ dy, const uint8_t* __restrict__ arg,
                                                              T* dx, int accumulate, int N, int H, int W, int C, int k,
                                                              int stride, int pad, int Ho, int Wo) {
    constexpr int VEC = Elem<T>::VEC;
    const int cv = C / VEC;
    const int64_t total = (int64_t)N * H * W * cv;
    const int64_t step = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += step) {
        const int c0 = (int)(i % cv) * VEC;
        int64_t t = i / cv;
        const int w = (int)(t % W); t /= W;
        const int h = (int)(t % H);
        const int n = (int)(t / H);
        float g[VEC];
        #pragma unroll
        for (int e = 0; e < VEC; ++e) g[e] = 0.f;
        for (int r = 0; r < k; ++r) {
            const int hn = h + pad - r;
            if (hn < 0 || hn % stride) continue;
            const int ho = hn / stride;
            if (ho >= Ho) continue;
            for (int s = 0; s < k; ++s) {
                const int wn = w + pad - s;
                if (wn < 0 || wn % stride) continue;
                const int wo = wn / stride;
                if (wo >= Wo) continue;
                const int64_t o = (((int64_t)n * Ho + ho) * Wo + wo) * C + c0;
                const Vec16<T> v = load_vec(dy + o);
                uint8_t am[VEC];
                if (VEC == 8) *reinterpret_cast<uint2*>(am) = *reinterpret_cast<const uint2*>(arg + o);
                else *reinterpret_cast<uint32_t*>(am) = *reinterpret_cast<const uint32_t*>(arg + o);
                #pragma unroll
                for (int e = 0; e < VEC; ++e)
                    if (am[e] == r * k + s) g[e] += Elem<T>::to_f32(v.e[e]);
            }
        }
        const int64_t xo = (((int64_t)n * H + h) * W + w) * C + c0;
        if (accumulate) {
            const Vec16<T> old = load_vec(dx + xo);
            #pragma unroll
            for (int e = 0; e < VEC; ++e) g[e] += Elem<T>::to_f32(old.e[e]);
        }
        Vec16<T> out;
        #pragma unroll
        for (int e = 0; e < VEC; ++e) out.e[e] = Elem<T>::from_f32(g[e]);
        store_vec(dx + xo, out);
    }
}

// The same with the window positions that can reach an input pixel enumerated without branches: at most
// NC = ceil(k / stride) per dimension.  All NC*NC loads are issued before the first use (a position outside
// the output reads a clamped one and is ignored), instead of one load and one wait per tap.
// MASK: the pooled tensor is the output of a ReLU; the gradient is stored already multiplied by (act > 0),
// so that the producer's backward need not read its activation again.
template <typename T, int NC, bool MASK>
__global__ __launch_bounds__(256) void maxpool_bwd_win_kernel(const T* __restrict__ dy, const uint8_t* __restrict__ arg,
                                                              T* dx, const T* __restrict__ act, int accumulate, int N, int H,
                                                              int W, int C, int k, int stride, int pad, int Ho, int Wo) {
    constexpr int VEC = Elem<T>::VEC;
    const int cv = C / VEC;
    const int64_t total = (int64_t)N * H * W * cv;
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    const int c0 = (int)(i % cv) * VEC;
    int64_t t = i / cv;
    const int w = (int)(t % W); t /= W;
    const int h = (int)(t % H);
    const int n = (int)(t / H);
    // output rows ho with ho*stride - pad <= h < ho*stride - pad + k: ho in [ho_hi - NC + 1, ho_hi]
    const int ho_hi = (h + pad) / stride, wo_hi = (w + pad) / stride;
    Vec16<T> v[NC][NC];
    uint8_t am[NC][NC][VEC];
    bool ok[NC][NC];
    int tap[NC][NC];
    #pragma unroll
    for (int a = 0; a < NC; ++a) {
        #pragma unroll
        for (int b = 0; b < NC; ++b) {
            const int ho = ho_hi - a, wo = wo_hi - b;
            const int r = h + pad - ho * stride, s2 = w + pad - wo * stride;      // tap of this pixel in that window
            ok[a][b] = ho >= 0 && wo >= 0 && ho < Ho && wo < Wo && r < k && s2 < k;
            tap[a][b] = r * k + s2;
            const int hc = ho < 0 ? 0 : (ho >= Ho ? Ho - 1 : ho), wc = wo < 0 ? 0 : (wo >= Wo ? Wo - 1 : wo);
            const int64_t o = (((int64_t)n * Ho + hc) * Wo + wc) * C + c0;
            v[a][b] = load_vec(dy + o);
            if (VEC == 8) *reinterpret_cast<uint2*>(am[a][b]) = *reinterpret_cast<const uint2*>(arg + o);
            else *reinterpret_cast<uint32_t*>(am[a][b]) = *reinterpret_cast<const uint32_t*>(arg + o);
        }
    }
    const int64_t xo = (((int64_t)n * H + h) * W + w) * C + c0;
    Vec16<T> old, av;
    old.u = make_uint4(0, 0, 0, 0);
    if (accumulate) old = load_vec(dx + xo);
    if (MASK) av = load_vec(act + xo);
    float g[VEC];
    #pragma unroll
    for (int e = 0; e < VEC; ++e) g[e] = 0.f;
    // taps in the order of the kernel above (r ascending, then s): the tap grows with a and b
    #pragma unroll
    for (int a = 0; a < NC; ++a) {
        #pragma unroll
        for (int b = 0; b < NC; ++b) {
            #pragma unroll
            for (int e = 0; e < VEC; ++e)
                if (ok[a][b] && am[a][b][e] == tap[a][b]) g[e] += Elem<T>::to_f32(v[a][b].e[e]);
        }
    }
    if (accumulate) {
        #pragma unroll
        for (int e = 0; e < VEC; ++e) g[e] += Elem<T>::to_f32(old.e[e]);
    }
    Vec16<T> out;
    #pragma unroll
    for (int e = 0; e < VEC; ++e) out.e[e] = Elem<T>::from_f32((!MASK || Elem<T>::to_f32(av.e[e]) > 0.f) ? g[e] : 0.f);
    store_vec(dx + xo, out);
}

void launch_maxpool_forward(int dtype, const void* x, void* y, uint8_t* arg, int N, int H, int W, int C, int k,
                            int stride, int pad, int Ho, int Wo, hipStream_t st) {
    const int grid = ew_grid((int64_t)N * Ho * Wo * C);
    const double esz = dtype == 1 ? 2.0 : 4.0;
    ProfScope ps("maxpool_fwd", 0.0, esz * (double)N * H * W * C + (esz + 1.0) * (double)N * Ho * Wo * C, st);
    const int vec = dtype == 1 ? 8 : 4;
    if (C % vec == 0) {
        const int vgrid = ew_grid((int64_t)N * Ho * Wo * (C / vec));
        if (dtype == 1)
            hipLaunchKernelGGL(maxpool_fwd_vec_kernel<bf16_t>, dim3(vgrid), dim3(256), 0, st, (const bf16_t*)x, (bf16_t*)y, arg,
                               N, H, W, C, k, stride, pad, Ho, Wo);
        else
            hipLaunchKernelGGL(maxpool_fwd_vec_kernel<float>, dim3(vgrid), dim3(256), 0, st, (const float*)x, (float*)y, arg, N,
                               H, W, C, k, stride, pad, Ho, Wo);
        return;
    }
    if (dtype == 1)
        hipLaunchKernelGGL(maxpool_fwd_kernel<bf16_t>, dim3(grid), dim3(256), 0, st, (const bf16_t*)x, (bf16_t*)y, arg, N,
                           H, W, C, k, stride, pad, Ho, Wo);
    else
        hipLaunchKernelGGL(maxpool_fwd_kernel<float>, dim3(grid), dim3(256), 0, st, (const float*)x, (float*)y, arg, N, H,
                           W, C, k, stride, pad, Ho, Wo);
}

bool launch_maxpool_backward(int dtype, const void* dy, const uint8_t* arg, void* dx, bool accumulate, int N, int H,
                             int W, int C, int k, int stride, int pad, int Ho, int Wo, const void* relu_act, hipStream_t st) {
    const int grid = ew_grid((int64_t)N * H * W * C);
    const double esz = dtype == 1 ? 2.0 : 4.0;
    const int vec = dtype == 1 ? 8 : 4;
    const int nc = (k + stride - 1) / stride;
    const int64_t lanes = C % vec == 0 ? (int64_t)N * H * W * (C / vec) : 0;
    const bool win = C % vec == 0 && nc <= 2 && lanes < (int64_t)1 << 38;
    const bool masked = win && relu_act != nullptr && !accumulate;
    ProfScope ps("maxpool_bwd", 0.0, esz * (double)N * H * W * C * ((accumulate ? 2.0 : 1.0) + (masked ? 1.0 : 0.0)) + (esz + 1.0) * (double)N * Ho * Wo * C, st);
    if (C % vec == 0) {
        const int vgrid = ew_grid((int64_t)N * H * W * (C / vec));
        if (win) {
            const dim3 g1((unsigned)((lanes + 255) / 256));
#define EDL_POOL_BWD(TT, NCC, MM)                                                                                               \
    hipLaunchKernelGGL((maxpool_bwd_win_kernel<TT, NCC, MM>), g1, dim3(256), 0, st, (const TT*)dy, arg, (TT*)dx, (const TT*)relu_act, \
                       accumulate ? 1 : 0, N, H, W, C, k, stride, pad, Ho, Wo)
            if (dtype == 1) {
                if (nc == 1) { if (masked) EDL_POOL_BWD(bf16_t, 1, true); else EDL_POOL_BWD(bf16_t, 1, false); }
                else { if (masked) EDL_POOL_BWD(bf16_t, 2, true); else EDL_POOL_BWD(bf16_t, 2, false); }
            } else {
                if (nc == 1) { if (masked) EDL_POOL_BWD(float, 1, true); else EDL_POOL_BWD(float, 1, false); }
                else { if (masked) EDL_POOL_BWD(float, 2, true); else EDL_POOL_BWD(float, 2, false); }
            }
#undef EDL_POOL_BWD
            return masked;
        }
        if (dtype == 1)
            hipLaunchKernelGGL(maxpool_bwd_vec_kernel<bf16_t>, dim3(vgrid), dim3(256), 0, st, (const bf16_t*)dy, arg,
                               (bf16_t*)dx, accumulate ? 1 : 0, N, H, W, C, k, stride, pad, Ho, Wo);
        else
            hipLaunchKernelGGL(maxpool_bwd_vec_kernel<float>, dim3(vgrid), dim3(256), 0, st, (const float*)dy, arg, (float*)dx,
                               accumulate ? 1 : 0, N, H, W, C, k, stride, pad, Ho, Wo);
        return false;
    }
    if (dtype == 1)
        hipLaunchKernelGGL(maxpool_bwd_kernel<bf16_t>, dim3(grid), dim3(256), 0, st, (const bf16_t*)dy, arg, (bf16_t*)dx,
                           accumulate ? 1 : 0, N, H, W, C, k, stride, pad, Ho, Wo);
    else
        hipLaunchKernelGGL(maxpool_bwd_kernel<float>, dim3(grid), dim3(256), 0, st, (const float*)dy, arg, (float*)dx,
                           accumulate ? 1 : 0, N, H, W, C, k, stride, pad, Ho, Wo);
    return false;
}

// ---------------------------------------------------------------------------
// global average pool: y[n][c] = mean over the HW pixels
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void gavgpool_fwd_kernel(const T* __restrict__ x, T* __restrict__ y, int N, int HW, int C) {
    const int64_t total = (int64_t)N * C;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const int c = (int)(i % C);
        const int64_t n = i / C;
        float s = 0.f;
        for (int q = 0; q < HW; ++q) s += Elem<T>::to_f32(x[(n * HW + q) * C + c]);
        y[i] = Elem<T>::from_f32(s / (float)HW);
    }
}

// The same on 16-byte vectors of channels: a block takes 64 channel vectors of one sample, its four
// quarter-blocks every fourth pixel each, and the four partial sums meet in LDS (a fixed order).
template <typename T>
__global__ __launch_bounds__(256) void gavgpool_fwd_vec_kernel(const T* __restrict__ x, T* __restrict__ y, int HW, int C) {
    constexpr int VEC = Elem<T>::VEC;
    __shared__ float part[3][64][VEC + 1];
    const int lane = threadIdx.x >> 6;
    const int cv = blockIdx.x * 64 + (threadIdx.x & 63);
    const int64_t n = blockIdx.y;
    const bool live = cv * VEC < C;
    float s[VEC];
#pragma unroll
    for (int j = 0; j < VEC; ++j) s[j] = 0.f;
    if (live) {
        const T* base = x + n * HW * C + (int64_t)cv * VEC;
#pragma unroll 4
        for (int q = lane; q < HW; q += 4) {
            const Vec16<T> v = load_vec(base + (int64_t)q * C);
#pragma unroll
            for (int j = 0; j < VEC; ++j) s[j] += Elem<T>::to_f32(v.e[j]);
        }
    }
    if (lane > 0) {
#pragma unroll
        for (int j = 0; j < VEC; ++j) part[lane - 1][threadIdx.x & 63][j] = s[j];
    }
    __syncthreads();
    if (lane == 0 && live) {
        Vec16<T> o;
#pragma unroll
        for (int j = 0; j < VEC; ++j) {
            const float t = ((s[j] + part[0][threadIdx.x][j]) + part[1][threadIdx.x][j]) + part[2][threadIdx.x][j];
            o.e[j] = Elem<T>::from_f32(t / (float)HW);
        }
        store_vec(y + n * C + (int64_t)cv * VEC, o);
    }
}

template <typename T>
__global__ __launch_bounds__(256) void gavgpool_bwd_kernel(const T* __restrict__ dy, T* dx, int accumulate, int N, int HW,
                                                           int C) {
    const int64_t total = (int64_t)N * HW * C;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const int c = (int)(i % C);
        const int64_t n = i / ((int64_t)HW * C);
        float g = Elem<T>::to_f32(dy[n * C + c]) / (float)HW;
        if (accumulate) g += Elem<T>::to_f32(dx[i]);
        dx[i] = Elem<T>::from_f32(g);
    }
}

void launch_gavgpool_forward(int dtype, const void* x, void* y, int N, int HW, int C, hipStream_t st) {
    const int grid = ew_grid((int64_t)N * C);
    ProfScope ps("gavgpool_fwd", 0.0, (dtype == 1 ? 2.0 : 4.0) * (double)N * (HW + 1) * C, st);
    const int vec = dtype == 1 ? 8 : 4;
    const bool aligned = ((uintptr_t)x | (uintptr_t)y) % 16 == 0;
    if (C % vec == 0 && aligned && N >= 1 && N <= 65535) {
        const dim3 vgrid((unsigned)((C / vec + 63) / 64), (unsigned)N);
        if (dtype == 1)
            hipLaunchKernelGGL(gavgpool_fwd_vec_kernel<bf16_t>, vgrid, dim3(256), 0, st, (const bf16_t*)x, (bf16_t*)y, HW, C);
        else
            hipLaunchKernelGGL(gavgpool_fwd_vec_kernel<float>, vgrid, dim3(256), 0, st, (const float*)x, (float*)y, HW, C);
    } else if (dtype == 1)
        hipLaunchKernelGGL(gavgpool_fwd_kernel<bf16_t>, dim3(grid), dim3(256), 0, st, (const bf16_t*)x, (bf16_t*)y, N, HW, C);
    else
        hipLaunchKernelGGL(gavgpool_fwd_kernel<float>, dim3(grid), dim3(256), 0, st, (const float*)x, (float*)y, N, HW, C);
}

void launch_gavgpool_backward(int dtype, const void* dy, void* dx, bool accumulate, int N, int HW, int C,
                              hipStream_t st) {
    const int grid = ew_grid((int64_t)N * HW * C);
    ProfScope ps("gavgpool_bwd", 0.0, (dtype == 1 ? 2.0 : 4.0) * (double)N * (HW + 1) * C, st);
    if (dtype == 1)
        hipLaunchKernelGGL(gavgpool_bwd_kernel<bf16_t>, dim3(grid), dim3(256), 0, st, (const bf16_t*)dy, (bf16_t*)dx,
                           accumulate ? 1 : 0, N, HW, C);
    else
        hipLaunchKernelGGL(gavgpool_bwd_kernel<float>, dim3(grid), dim3(256), 0, st, (const float*)dy, (float*)dx,
                           accumulate ? 1 : 0, N, HW, C);
}

// ---------------------------------------------------------------------------
// softmax cross-entropy: one workgroup per sample.  loss_i = log(sum exp(z -
// max)) - (z_label - max); dz = (softmax - onehot) / n.
// ---------------------------------------------------------------------------
__device__ __forceinline__ float block_reduce(float v, float* sm, bool is_max) {
    for (int o = 32; o > 0; o >>= 1) {
        const float other = __shfl_xor(v, o, 64);
        v = is_max ? fmaxf(v, other) : v + other;
    }
    const int wave = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sm[wave] = v;
    __syncthreads();
    float r = sm[0];
    for (int i = 1; i < (int)(blockDim.x >> 6); ++i) r = is_max ? fmaxf(r, sm[i]) : r + sm[i];
    return r;
}

template <typename T>
__global__ __launch_bounds__(256) void softmax_ce_kernel(const float* __restrict__ logits, const int32_t* __restrict__ labels,
                                                         T* __restrict__ dlogits, float* __restrict__ row_loss, int n, int C) {
    __shared__ float sm[4];
    const int i = blockIdx.x;
    const float* z = logits + (int64_t)i * C;
    float mx = -INFINITY;
    for (int c = threadIdx.x; c < C; c += blockDim.x) mx = fmaxf(mx, z[c]);
    mx = block_reduce(mx, sm, true);
    float s = 0.f;
    for (int c = threadIdx.x; c < C; c += blockDim.x) s += expf(z[c] - mx);
    s = block_reduce(s, sm, false);
    const int label = labels[i];
    const float inv = 1.f / s, invn = 1.f / (float)n;
    for (int c = threadIdx.x; c < C; c += blockDim.x) {
        const float pr = expf(z[c] - mx) * inv;
        dlogits[(int64_t)i * C + c] = Elem<T>::from_f32((pr - (c == label ? 1.f : 0.f)) * invn);
    }
    if (threadIdx.x == 0) row_loss[i] = logf(s) - (z[label] - mx);
}

// mean of the n per-sample losses, summed in sample order by one wave
__global__ void loss_mean_kernel(const float* __restrict__ row_loss, int n, float* __restrict__ out) {
    float s = 0.f;
    for (int i = threadIdx.x; i < n; i += 64) s += row_loss[i];
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
    if (threadIdx.x == 0) out[0] = s / (float)n;
}

void launch_softmax_ce(int dtype, const float* logits, const int32_t* labels, void* dlogits, float* row_loss,
                       float* loss_out, int n, int C, hipStream_t st) {
    ProfScope ps("softmax_ce", 0.0, (4.0 + (dtype == 1 ? 2.0 : 4.0)) * (double)n * C, st);
    if (dtype == 1)
        hipLaunchKernelGGL(softmax_ce_kernel<bf16_t>, dim3(n), dim3(256), 0, st, logits, labels, (bf16_t*)dlogits, row_loss, n, C);
    else
        hipLaunchKernelGGL(softmax_ce_kernel<float>, dim3(n), dim3(256), 0, st, logits, labels, (float*)dlogits, row_loss, n, C);
    hipLaunchKernelGGL(loss_mean_kernel, dim3(1), dim3(64), 0, st, row_loss, n, loss_out);
}

// ---------------------------------------------------------------------------
// Attainable matrix rate: every wave keeps four independent 32x32 accumulators
// and issues MFMAs on register operands only (no memory in the loop).  What the
// convolutions' MFMA fractions can be held against besides the data sheet.
// ---------------------------------------------------------------------------
typedef float mfma_acc_t __attribute__((ext_vector_type(16)));
typedef __bf16 mfma_bf16x8_t __attribute__((ext_vector_type(8)));

template <bool BF16>
__global__ __launch_bounds__(256) void mfma_rate_kernel(int iters, float* __restrict__ sink) {
    mfma_acc_t acc[4];
    #pragma unroll
    for (int q = 0; q < 4; ++q)
        #pragma unroll
        for (int e = 0; e < 16; ++e) acc[q][e] = 0.f;
    const float seed = 1.0f + (float)(threadIdx.x & 7) * 0.125f;
    mfma_bf16x8_t a, b;
    #pragma unroll
    for (int e = 0; e < 8; ++e) { a[e] = (__bf16)seed; b[e] = (__bf16)(1.0f / seed); }
    for (int i = 0; i < iters; ++i) {
        #pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (BF16) acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[q], 0, 0, 0);
            else acc[q] = __builtin_amdgcn_mfma_f32_32x32x2f32(seed, 1.0f / seed, acc[q], 0, 0, 0);
        }
    }
    float t = 0.f;
    #pragma unroll
    for (int q = 0; q < 4; ++q)
        #pragma unroll
        for (int e = 0; e < 16; ++e) t += acc[q][e];
    if (t == 12345.678f) sink[0] = t;   // never true; keeps the accumulators alive
}

// flops issued: blocks * 4 waves * iters * 4 MFMAs * 2*32*32*k
double launch_mfma_rate(int dtype, int blocks, int iters, float* sink, hipStream_t st) {
    const double per_mfma = dtype == 1 ? 2.0 * 32 * 32 * 16 : 2.0 * 32 * 32 * 2;
    const double flops = (double)blocks * 4.0 * (double)iters * 4.0 * per_mfma;
    ProfScope ps(dtype == 1 ? "mfma_rate_bf16" : "mfma_rate_f32", flops, 0.0, st);
    if (dtype == 1) hipLaunchKernelGGL(mfma_rate_kernel<true>, dim3(blocks), dim3(256), 0, st, iters, sink);
    else hipLaunchKernelGGL(mfma_rate_kernel<false>, dim3(blocks), dim3(256), 0, st, iters, sink);
    return flops;
}

}  // namespace edl
