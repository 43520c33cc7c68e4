// HBM-bound kernels of the step: aggregation of the workers' gradients fused
// with the momentum-SGD update (the all-reduce + optimizer of section 2.1 on
// one GPU), the state copy a joining worker receives (section 4.2), and the
// sample gather that stands for the prefetch pipeline (section 4.4).
#include <algorithm>
#include <cstdlib>

#include "dev_common.h"
#include "kernels.h"
#include "profiler.h"
#include "tune.h"

namespace edl {

static inline int grid_for(int64_t work_items, int block, int max_blocks) {
    int64_t b = (work_items + block - 1) / block;
    if (b < 1) b = 1;
    if (b > max_blocks) b = max_blocks;
    return (int)b;
}

// ---------------------------------------------------------------------------
// g = (sum_k G_k)/p + wd*w ; v = momentum*v + g ; w = w - lr*v ; w16 = bf16(w)
// One 16-byte vector per lane per stream; p+2 read streams and 2 (+1) write
// streams, all fully coalesced.  NP > 0 fixes p at compile time so that all
// p loads are in flight together.
// ---------------------------------------------------------------------------
// One lane handles VPT consecutive 16-byte vectors of every stream.
template <int NP, bool SHADOW, int VPT>
__global__ __launch_bounds__(256) void average_update_kernel(GradPtrs gp, int p, float* __restrict__ w,
                                                             float* __restrict__ v, uint16_t* __restrict__ w16,
                                                             int64_t nvec, int64_t P, float lr, float momentum,
                                                             float wd) {
    const int np = NP > 0 ? NP : p;
    const float fp = (float)np;
    // one pass for a launch that covers the vector (the usual one); a launch held to fewer workgroups, which
    // runs in the background of other work, strides on
    const int64_t step = (int64_t)gridDim.x * blockDim.x * VPT;
    for (int64_t i0 = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * VPT; i0 < nvec; i0 += step) {
        float4 s[VPT], wi[VPT], vi[VPT];
        #pragma unroll
        for (int u = 0; u < VPT; ++u) {
            const int64_t i = i0 + u < nvec ? i0 + u : nvec - 1;     // the last lane may repeat a vector (same result)
            s[u] = reinterpret_cast<const float4*>(gp.g[0])[i];
            wi[u] = reinterpret_cast<float4*>(w)[i];
            vi[u] = reinterpret_cast<float4*>(v)[i];
        }
        if (NP > 0) {
            #pragma unroll
            for (int k = 1; k < NP; ++k) {
                #pragma unroll
                for (int u = 0; u < VPT; ++u) {
                    const int64_t i = i0 + u < nvec ? i0 + u : nvec - 1;
                    const float4 t = reinterpret_cast<const float4*>(gp.g[k])[i];
                    s[u].x += t.x; s[u].y += t.y; s[u].z += t.z; s[u].w += t.w;
                }
            }
        } else {
            for (int k = 1; k < np; ++k) {
                #pragma unroll
                for (int u = 0; u < VPT; ++u) {
                    const int64_t i = i0 + u < nvec ? i0 + u : nvec - 1;
                    const float4 t = reinterpret_cast<const float4*>(gp.g[k])[i];
                    s[u].x += t.x; s[u].y += t.y; s[u].z += t.z; s[u].w += t.w;
                }
            }
        }
        #pragma unroll
        for (int u = 0; u < VPT; ++u) {
            if (i0 + u >= nvec) break;
            const int64_t i = i0 + u;
            vi[u].x = momentum * vi[u].x + (s[u].x / fp + wd * wi[u].x);
            vi[u].y = momentum * vi[u].y + (s[u].y / fp + wd * wi[u].y);
            vi[u].z = momentum * vi[u].z + (s[u].z / fp + wd * wi[u].z);
            vi[u].w = momentum * vi[u].w + (s[u].w / fp + wd * wi[u].w);
            wi[u].x -= lr * vi[u].x; wi[u].y -= lr * vi[u].y; wi[u].z -= lr * vi[u].z; wi[u].w -= lr * vi[u].w;
            reinterpret_cast<float4*>(v)[i] = vi[u];
            reinterpret_cast<float4*>(w)[i] = wi[u];
            if (SHADOW) reinterpret_cast<uint2*>(w16)[i] = make_uint2(pack2_bf16(wi[u].x, wi[u].y), pack2_bf16(wi[u].z, wi[u].w));
        }
    }
    // ragged tail (P not a multiple of 4): the first few lanes of block 0
    if (blockIdx.x == 0 && threadIdx.x < (unsigned)(P - nvec * 4)) {
        const int64_t i = nvec * 4 + threadIdx.x;
        float s = gp.g[0][i];
        for (int k = 1; k < np; ++k) s += gp.g[k][i];
        float wi = w[i];
        const float vi = momentum * v[i] + (s / fp + wd * wi);
        wi -= lr * vi;
        v[i] = vi;
        w[i] = wi;
        if (SHADOW) w16[i] = f32_to_bf16(wi);
    }
}

// The same update with the streams walked in wave-wide pieces: a workgroup owns U * 256 consecutive vectors of
// every stream and lane t takes vectors t, t + 256, ... of them, so each of the workgroup's load instructions
// covers 4 KB of one stream and all (NP + 2) * U loads of a lane are in flight before the first is used.  NT bit 0:
// the gradient buffers (read once, never again) are loaded non-temporally; bit 1: so is the bf16 copy stored.
// Same arithmetic in the same order as average_update_kernel: the results are bit-identical.
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

template <int NP, bool SHADOW, int U, int NT>
__global__ __launch_bounds__(256) void average_update_wide_kernel(GradPtrs gp, float* __restrict__ w, float* __restrict__ v,
                                                                  uint16_t* __restrict__ w16, int64_t nvec, int64_t P, float lr,
                                                                  float momentum, float wd) {
    const float fp = (float)NP;
    const int64_t step = (int64_t)gridDim.x * 256 * U;
    for (int64_t i0 = (int64_t)blockIdx.x * 256 * U + threadIdx.x; i0 - threadIdx.x < nvec; i0 += step) {
        f32x4 s[U], wi[U], vi[U];
        #pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = i0 + u * 256 < nvec ? i0 + u * 256 : nvec - 1;     // lanes past the end repeat the last vector
            const f32x4* g0 = reinterpret_cast<const f32x4*>(gp.g[0]) + i;
            s[u] = (NT & 1) ? __builtin_nontemporal_load(g0) : *g0;
            const f32x4* wp = reinterpret_cast<const f32x4*>(w) + i;
            const f32x4* vp = reinterpret_cast<const f32x4*>(v) + i;
            wi[u] = (NT & 4) ? __builtin_nontemporal_load(wp) : *wp;
            vi[u] = (NT & 4) ? __builtin_nontemporal_load(vp) : *vp;
        }
        #pragma unroll
        for (int k = 1; k < NP; ++k) {
            f32x4 t[U];
            #pragma unroll
            for (int u = 0; u < U; ++u) {
                const int64_t i = i0 + u * 256 < nvec ? i0 + u * 256 : nvec - 1;
                const f32x4* gk = reinterpret_cast<const f32x4*>(gp.g[k]) + i;
                t[u] = (NT & 1) ? __builtin_nontemporal_load(gk) : *gk;
            }
            #pragma unroll
            for (int u = 0; u < U; ++u) s[u] += t[u];
        }
        #pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = i0 + u * 256;
            if (i >= nvec) break;
            f32x4 vn, wn;
            #pragma unroll
            for (int e = 0; e < 4; ++e) {
                vn[e] = momentum * vi[u][e] + (s[u][e] / fp + wd * wi[u][e]);
                wn[e] = wi[u][e] - lr * vn[e];
            }
            if (NT & 4) {
                __builtin_nontemporal_store(vn, reinterpret_cast<f32x4*>(v) + i);
                __builtin_nontemporal_store(wn, reinterpret_cast<f32x4*>(w) + i);
            } else {
                reinterpret_cast<f32x4*>(v)[i] = vn;
                reinterpret_cast<f32x4*>(w)[i] = wn;
            }
            if (SHADOW) {
                const u32x2 packed = {pack2_bf16(wn[0], wn[1]), pack2_bf16(wn[2], wn[3])};
                if (NT & 2) __builtin_nontemporal_store(packed, reinterpret_cast<u32x2*>(w16) + i);
                else reinterpret_cast<u32x2*>(w16)[i] = packed;
            }
        }
    }
    // ragged tail (P not a multiple of 4): the first few lanes of block 0
    if (blockIdx.x == 0 && threadIdx.x < (unsigned)(P - nvec * 4)) {
        const int64_t i = nvec * 4 + threadIdx.x;
        float s = gp.g[0][i];
        for (int k = 1; k < NP; ++k) s += gp.g[k][i];
        float wi = w[i];
        const float vi = momentum * v[i] + (s / fp + wd * wi);
        wi -= lr * vi;
        v[i] = vi;
        w[i] = wi;
        if (SHADOW) w16[i] = f32_to_bf16(wi);
    }
}

template <int NP, int U, int NT>
static void launch_update_wide(int grid, const GradPtrs& grads, float* w, float* v, uint16_t* w16, int64_t nvec, int64_t P,
                               float lr, float momentum, float wd, hipStream_t st) {
    if (w16) hipLaunchKernelGGL((average_update_wide_kernel<NP, true, U, NT>), dim3(grid), dim3(256), 0, st, grads, w, v, w16, nvec, P, lr, momentum, wd);
    else hipLaunchKernelGGL((average_update_wide_kernel<NP, false, U, NT>), dim3(grid), dim3(256), 0, st, grads, w, v, w16, nvec, P, lr, momentum, wd);
}

template <int NP>
static bool launch_update_wide_np(int u, int nt, int grid, const GradPtrs& grads, float* w, float* v, uint16_t* w16, int64_t nvec,
                                  int64_t P, float lr, float momentum, float wd, hipStream_t st) {
#define EDL_WIDE(U_, NT_) if (u == U_ && nt == NT_) { launch_update_wide<NP, U_, NT_>(grid, grads, w, v, w16, nvec, P, lr, momentum, wd, st); return true; }
    EDL_WIDE(1, 0) EDL_WIDE(1, 1) EDL_WIDE(1, 3) EDL_WIDE(1, 7) EDL_WIDE(2, 0) EDL_WIDE(2, 3) EDL_WIDE(2, 7) EDL_WIDE(4, 0) EDL_WIDE(4, 3) EDL_WIDE(4, 7)
#undef EDL_WIDE
    return false;
}

template <int NP, int VPT>
static void launch_update_t(int grid, const GradPtrs& grads, int p, float* w, float* v, uint16_t* w16, int64_t nvec, int64_t P,
                            float lr, float momentum, float wd, hipStream_t st) {
    if (w16) hipLaunchKernelGGL((average_update_kernel<NP, true, VPT>), dim3(grid), dim3(256), 0, st, grads, p, w, v, w16, nvec, P, lr, momentum, wd);
    else hipLaunchKernelGGL((average_update_kernel<NP, false, VPT>), dim3(grid), dim3(256), 0, st, grads, p, w, v, w16, nvec, P, lr, momentum, wd);
}

void launch_average_update(int p, const GradPtrs& grads, float* w, float* v, uint16_t* w16, int64_t P, float lr,
                           float momentum, float wd, hipStream_t st, int max_blocks) {
    const int64_t nvec = P / 4;
    // one workgroup per 256*VPT vectors, no grid-stride loop (measured ~20% faster than looping over a few thousand workgroups)
    const int vpt = (int)tune().upd_vpt;
    const int64_t per_block = 256 * (vpt == 2 ? 2 : 1);
    int grid = (int)std::max<int64_t>(1, (nvec + per_block - 1) / per_block);
    if (max_blocks > 0 && grid > max_blocks) grid = max_blocks;
    // p gradient reads + w, v read and written (+ the bf16 copy)
    ProfScope ps("average_update", 0.0, (4.0 * p + 16.0 + (w16 ? 2.0 : 0.0)) * (double)P, st);
#define EDL_UPD(NP)                                                                                   \
    do {                                                                                              \
        if (vpt == 2) launch_update_t<NP, 2>(grid, grads, p, w, v, w16, nvec, P, lr, momentum, wd, st); \
        else launch_update_t<NP, 1>(grid, grads, p, w, v, w16, nvec, P, lr, momentum, wd, st);          \
    } while (0)
    // the wave-wide walk (upd_wide = vectors per lane, 0 = the kernel above, -1 = by p), upd_nt = non-temporal flags
    // (-1 = by p), upd_blocks > 0 = a grid-stride launch of that many workgroups
    // Measured on the 138 M-parameter state (update sweep, MI355X): the wave-wide walk with non-temporal
    // gradient loads and bf16 store gives 5.9 / 5.7 / 5.7 TB/s at p = 1 / 2 / 4 with one vector per lane (the kernel
    // above: 5.4 / 5.3 / 5.2), and 5.6 TB/s at p = 8 with four vectors per lane and w, v non-temporal too (5.3).
    // Where w and v start on 4 KB boundaries of opposite parity (address bit 12; the library's own arena
    // alternates it from one state array to the next), their pieces no longer meet in the same half of the
    // memory system at the same moment, and one vector per lane is the best walk for every p.  At the end of
    // a VGG-16 training step: 6.4 / 6.3 / 6.1 / 5.9 TB/s at p = 1 / 2 / 4 / 8 with non-temporal gradient loads and
    // bf16 store (w, v non-temporal as well: 6.2 / 6.2 / 6.1 / 5.9; four vectors per lane: 5.7).  Launched back to
    // back on its own, the same kernel reads 6.0 / 5.9 / 5.9 / 5.8 (on arrays that all start on 8 KB boundaries
    // 5.8 / 5.5 / 5.6 / 5.6): the previous launch's stores are still being written back.
    // (a piece of the arrays that starts at the same offset of both keeps that relation: same position inside the
    // page, pages of opposite parity)
    const uintptr_t wv = (uintptr_t)w ^ (uintptr_t)v;
    const bool alternating = (wv & 4095) == 0 && ((wv >> 12) & 1) != 0;
    int wide = (int)tune().upd_wide, nt = (int)tune().upd_nt;
    if (wide < 0) wide = alternating ? 1 : p >= 8 ? 4 : 1;
    if (nt < 0) nt = alternating ? 3 : p >= 8 ? 7 : 3;
    if (wide > 0 && (p == 1 || p == 2 || p == 4 || p == 8)) {
        int wgrid = (int)std::max<int64_t>(1, (nvec + 256 * wide - 1) / (256 * wide));
        if (tune().upd_blocks > 0 && wgrid > tune().upd_blocks) wgrid = (int)tune().upd_blocks;
        if (max_blocks > 0 && wgrid > max_blocks) wgrid = max_blocks;
        bool done = false;
        switch (p) {
            case 1: done = launch_update_wide_np<1>(wide, nt, wgrid, grads, w, v, w16, nvec, P, lr, momentum, wd, st); break;
            case 2: done = launch_update_wide_np<2>(wide, nt, wgrid, grads, w, v, w16, nvec, P, lr, momentum, wd, st); break;
            case 4: done = launch_update_wide_np<4>(wide, nt, wgrid, grads, w, v, w16, nvec, P, lr, momentum, wd, st); break;
            default: done = launch_update_wide_np<8>(wide, nt, wgrid, grads, w, v, w16, nvec, P, lr, momentum, wd, st); break;
        }
        if (done) return;
    }
    switch (p) {
        case 1: EDL_UPD(1); break;
        case 2: EDL_UPD(2); break;
        case 4: EDL_UPD(4); break;
        case 8: EDL_UPD(8); break;
        default: EDL_UPD(0); break;
    }
#undef EDL_UPD
}

// The same for shards of unequal size: the aggregate is sum_k share[k] * G_k, share[k] = the shard's
// part of the mini-batch (section 2.1: the mean of the per-sample gradients of the mini-batch).  Rare (a tail
// mini-batch of the data pipeline, a mini-batch redone by the survivors of a failure): one element per lane.
template <bool SHADOW>
__global__ __launch_bounds__(256) void weighted_update_kernel(GradPtrs gp, ShardShares sh, int np, float* __restrict__ w,
                                                              float* __restrict__ v, uint16_t* __restrict__ w16, int64_t P,
                                                              float lr, float momentum, float wd) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= P) return;
    float s = sh.share[0] * gp.g[0][i];
    for (int k = 1; k < np; ++k) s += sh.share[k] * gp.g[k][i];
    float wi = w[i];
    const float vi = momentum * v[i] + (s + wd * wi);
    wi -= lr * vi;
    v[i] = vi;
    w[i] = wi;
    if (SHADOW) w16[i] = f32_to_bf16(wi);
}

void launch_weighted_update(int np, const GradPtrs& grads, const ShardShares& shares, float* w, float* v, uint16_t* w16,
                            int64_t P, float lr, float momentum, float wd, hipStream_t st) {
    const int grid = (int)((P + 255) / 256);
    ProfScope ps("weighted_update", 0.0, (4.0 * np + 16.0 + (w16 ? 2.0 : 0.0)) * (double)P, st);
    if (w16) hipLaunchKernelGGL(weighted_update_kernel<true>, dim3(grid), dim3(256), 0, st, grads, shares, np, w, v, w16, P, lr, momentum, wd);
    else hipLaunchKernelGGL(weighted_update_kernel<false>, dim3(grid), dim3(256), 0, st, grads, shares, np, w, v, w16, P, lr, momentum, wd);
}

// ---------------------------------------------------------------------------
// Adam on the aggregated gradient (the optimizer of the usage example in
// section 3.2; steps of Algorithm 1 of Kingma & Ba):
//   g = aggregate + wd*w ; m = b1*m + (1-b1)*g ; s = b2*s + (1-b2)*g*g ;
//   w = w - lr * (m*c1) / (sqrt(s*c2) + eps) ; w16 = bf16(w)
// with c1 = 1/(1-b1^t), c2 = 1/(1-b2^t) formed by the host.  p+3 read streams,
// 3 (+1) write streams, one 16-byte vector per lane per stream.  NP > 0 fixes p
// at compile time (all p loads in flight); WEIGHTED takes sum_k share[k]*G_k
// instead of the mean.
// ---------------------------------------------------------------------------
struct AdamCoef { float lr, b1, b2, eps, wd, c1, c2; };

__device__ __forceinline__ void adam_one(float g, float& w, float& m, float& s, const AdamCoef& a) {
    g += a.wd * w;
    m = a.b1 * m + (1.0f - a.b1) * g;
    s = a.b2 * s + (1.0f - a.b2) * (g * g);
    w -= a.lr * (m * a.c1) / (sqrtf(s * a.c2) + a.eps);
}

template <int NP, bool WEIGHTED, bool SHADOW>
__global__ __launch_bounds__(256) void adam_update_kernel(GradPtrs gp, ShardShares sh, int p, float* __restrict__ w,
                                                          float* __restrict__ m, float* __restrict__ s,
                                                          uint16_t* __restrict__ w16, int64_t nvec, int64_t P, AdamCoef a) {
    const int np = NP > 0 ? NP : p;
    const float inv_p = 1.0f / (float)np;
    const int64_t step = (int64_t)gridDim.x * blockDim.x;   // see average_update_kernel
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < nvec; i += step) {
        float4 wi = reinterpret_cast<float4*>(w)[i];
        float4 mi = reinterpret_cast<float4*>(m)[i];
        float4 si = reinterpret_cast<float4*>(s)[i];
        // the gradient buffers are read once and never again: non-temporal loads (as is the bf16 store below)
        const f32x4 g0 = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(gp.g[0]) + i);
        float4 g = make_float4(g0[0], g0[1], g0[2], g0[3]);
        if (WEIGHTED) { g.x *= sh.share[0]; g.y *= sh.share[0]; g.z *= sh.share[0]; g.w *= sh.share[0]; }
        if (NP > 0) {
            f32x4 t[NP > 1 ? NP - 1 : 1];
            #pragma unroll
            for (int k = 1; k < NP; ++k) t[k - 1] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(gp.g[k]) + i);
            #pragma unroll
            for (int k = 1; k < NP; ++k) {
                const float c = WEIGHTED ? sh.share[k] : 1.0f;
                g.x += c * t[k - 1][0]; g.y += c * t[k - 1][1]; g.z += c * t[k - 1][2]; g.w += c * t[k - 1][3];
            }
        } else {
            for (int k = 1; k < np; ++k) {
                const f32x4 t = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(gp.g[k]) + i);
                const float c = WEIGHTED ? sh.share[k] : 1.0f;
                g.x += c * t[0]; g.y += c * t[1]; g.z += c * t[2]; g.w += c * t[3];
            }
        }
        if (!WEIGHTED) { g.x *= inv_p; g.y *= inv_p; g.z *= inv_p; g.w *= inv_p; }
        adam_one(g.x, wi.x, mi.x, si.x, a);
        adam_one(g.y, wi.y, mi.y, si.y, a);
        adam_one(g.z, wi.z, mi.z, si.z, a);
        adam_one(g.w, wi.w, mi.w, si.w, a);
        reinterpret_cast<float4*>(m)[i] = mi;
        reinterpret_cast<float4*>(s)[i] = si;
        reinterpret_cast<float4*>(w)[i] = wi;
        if (SHADOW) {
            const u32x2 packed = {pack2_bf16(wi.x, wi.y), pack2_bf16(wi.z, wi.w)};
            __builtin_nontemporal_store(packed, reinterpret_cast<u32x2*>(w16) + i);
        }
    }
    // ragged tail (P not a multiple of 4): the first few lanes of block 0
    if (blockIdx.x == 0 && threadIdx.x < (unsigned)(P - nvec * 4)) {
        const int64_t j = nvec * 4 + threadIdx.x;
        float g = gp.g[0][j] * (WEIGHTED ? sh.share[0] : 1.0f);
        for (int k = 1; k < np; ++k) g += gp.g[k][j] * (WEIGHTED ? sh.share[k] : 1.0f);
        if (!WEIGHTED) g *= inv_p;
        float wj = w[j], mj = m[j], sj = s[j];
        adam_one(g, wj, mj, sj, a);
        m[j] = mj; s[j] = sj; w[j] = wj;
        if (SHADOW) w16[j] = f32_to_bf16(wj);
    }
}

template <int NP, bool WEIGHTED>
static void launch_adam_t(int grid, const GradPtrs& grads, const ShardShares& sh, int p, float* w, float* m, float* s,
                          uint16_t* w16, int64_t nvec, int64_t P, const AdamCoef& a, hipStream_t st) {
    if (w16) hipLaunchKernelGGL((adam_update_kernel<NP, WEIGHTED, true>), dim3(grid), dim3(256), 0, st, grads, sh, p, w, m, s, w16, nvec, P, a);
    else hipLaunchKernelGGL((adam_update_kernel<NP, WEIGHTED, false>), dim3(grid), dim3(256), 0, st, grads, sh, p, w, m, s, w16, nvec, P, a);
}

void launch_adam_update(int p, const GradPtrs& grads, const ShardShares* shares, float* w, float* m, float* s, uint16_t* w16,
                        int64_t P, float lr, float beta1, float beta2, float eps, float wd, float c1, float c2, hipStream_t st,
                        int max_blocks) {
    const int64_t nvec = P / 4;
    int grid = (int)std::max<int64_t>(1, (nvec + 255) / 256);
    if (max_blocks > 0 && grid > max_blocks) grid = max_blocks;
    const AdamCoef a = {lr, beta1, beta2, eps, wd, c1, c2};
    // p gradient reads + w, m, s read and written (+ the bf16 copy)
    ProfScope ps("adam_update", 0.0, (4.0 * p + 24.0 + (w16 ? 2.0 : 0.0)) * (double)P, st);
    const ShardShares none = {};
    if (shares) {
        launch_adam_t<0, true>(grid, grads, *shares, p, w, m, s, w16, nvec, P, a, st);
        return;
    }
    switch (p) {
        case 1: launch_adam_t<1, false>(grid, grads, none, p, w, m, s, w16, nvec, P, a, st); break;
        case 2: launch_adam_t<2, false>(grid, grads, none, p, w, m, s, w16, nvec, P, a, st); break;
        case 4: launch_adam_t<4, false>(grid, grads, none, p, w, m, s, w16, nvec, P, a, st); break;
        case 8: launch_adam_t<8, false>(grid, grads, none, p, w, m, s, w16, nvec, P, a, st); break;
        default: launch_adam_t<0, false>(grid, grads, none, p, w, m, s, w16, nvec, P, a, st); break;
    }
}

// ---------------------------------------------------------------------------
// plain copy (snapshot / restore): 16-byte vectors when source, destination
// and length allow it (the large state arrays do), else 4-byte or 1-byte units
// ---------------------------------------------------------------------------
template <typename U>
__global__ __launch_bounds__(256) void copy_kernel(U* __restrict__ dst, const U* __restrict__ src, int64_t n) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

void launch_copy(void* dst, const void* src, size_t bytes, hipStream_t st) {
    if (bytes == 0) return;
    ProfScope ps("copy", 0.0, 2.0 * (double)bytes, st);
    const uintptr_t bits = (uintptr_t)dst | (uintptr_t)src | (uintptr_t)bytes;
    if ((bits & 15) == 0) {
        const int64_t n = (int64_t)(bytes / 16);
        hipLaunchKernelGGL(copy_kernel<uint4>, dim3(grid_for(n, 256, 1 << 30)), dim3(256), 0, st, (uint4*)dst, (const uint4*)src, n);
    } else if ((bits & 3) == 0) {
        const int64_t n = (int64_t)(bytes / 4);
        hipLaunchKernelGGL(copy_kernel<uint32_t>, dim3(grid_for(n, 256, 1 << 30)), dim3(256), 0, st, (uint32_t*)dst, (const uint32_t*)src, n);
    } else {
        const int64_t n = (int64_t)bytes;
        hipLaunchKernelGGL(copy_kernel<uint8_t>, dim3(grid_for(n, 256, 1 << 30)), dim3(256), 0, st, (uint8_t*)dst, (const uint8_t*)src, n);
    }
}

__global__ __launch_bounds__(256) void fill_kernel(float* dst, float value, int64_t n) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = value;
}

void launch_fill_f32(float* dst, float value, int64_t n, hipStream_t st) {
    if (n <= 0) return;
    ProfScope ps("fill", 0.0, 4.0 * (double)n, st);
    hipLaunchKernelGGL(fill_kernel, dim3(grid_for(n, 256, 4096)), dim3(256), 0, st, dst, value, n);
}

__global__ __launch_bounds__(256) void cast_bf16_kernel(const float* __restrict__ src, uint16_t* __restrict__ dst,
                                                        int64_t n) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = f32_to_bf16(src[i]);
}

void launch_cast_bf16(const float* src, uint16_t* dst, int64_t n, hipStream_t st) {
    if (n <= 0) return;
    ProfScope ps("cast_bf16", 0.0, 6.0 * (double)n, st);
    hipLaunchKernelGGL(cast_bf16_kernel, dim3(grid_for(n, 256, 4096)), dim3(256), 0, st, src, dst, n);
}

// ---------------------------------------------------------------------------
// dst[c][t][k] = cast(src[k][t][c]),  t = kernel tap.  32x32 tiles through LDS
// so that both the read (c innermost) and the write (k innermost) coalesce.
// ---------------------------------------------------------------------------
// All layers in one launch: workgroup b finds its layer in the table by its
// first-tile index, then transposes one 32x32 tile of one tap.
template <typename T>
__global__ __launch_bounds__(256) void weight_transpose_all_kernel(const float* __restrict__ w, unsigned char* __restrict__ arena,
                                                                   const TransposeEntry* __restrict__ tab, int entries) {
    __shared__ float tile[32][33];
    int e = 0, hi = entries - 1;   // last entry whose first tile is not beyond this workgroup's
    while (e < hi) {
        const int mid = (e + hi + 1) >> 1;
        if ((int)blockIdx.x >= tab[mid].tile_start) e = mid;
        else hi = mid - 1;
    }
    const TransposeEntry te = tab[e];
    int b = blockIdx.x - te.tile_start;
    const int tiles_c = (te.C + 31) / 32, tiles_k = (te.K + 31) / 32;
    const int cx = b % tiles_c; b /= tiles_c;
    const int ky = b % tiles_k;
    const int t = b / tiles_k;
    const float* src = w + te.src_off;
    T* dst = reinterpret_cast<T*>(arena + te.dst_off);
    const int c0 = cx * 32, k0 = ky * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    for (int i = ty; i < 32; i += 8) {
        const int k = k0 + i, c = c0 + tx;
        tile[i][tx] = (k < te.K && c < te.C) ? src[((int64_t)k * te.RS + t) * te.C + c] : 0.f;
    }
    __syncthreads();
    for (int i = ty; i < 32; i += 8) {
        const int c = c0 + i, k = k0 + tx;
        if (c < te.C && k < te.K) dst[((int64_t)c * te.RS + t) * te.K + k] = Elem<T>::from_f32(tile[tx][i]);
    }
}

// The same for bf16 layers whose K and C are multiples of 8, from the bf16 copy of the weights (two bytes
// read per element instead of four): 64x64 tiles, 16-byte loads and stores.  tile_start counts 64x64 tiles.
__global__ __launch_bounds__(256) void weight_transpose_bf16_kernel(const uint16_t* __restrict__ w16, unsigned char* __restrict__ arena,
                                                                    const TransposeEntry* __restrict__ tab, int entries) {
    constexpr int LD = 68;   // elements per tile row in LDS: rows 8-byte aligned, column reads spread over the banks
    __shared__ __attribute__((aligned(16))) uint16_t tile[64 * LD];
    int e = 0, hi = entries - 1;
    while (e < hi) {
        const int mid = (e + hi + 1) >> 1;
        if ((int)blockIdx.x >= tab[mid].tile_start) e = mid;
        else hi = mid - 1;
    }
    const TransposeEntry te = tab[e];
    int b = blockIdx.x - te.tile_start;
    const int tiles_c = (te.C + 63) / 64, tiles_k = (te.K + 63) / 64;
    const int cx = b % tiles_c; b /= tiles_c;
    const int ky = b % tiles_k;
    const int t = b / tiles_k;
    const uint16_t* src = w16 + te.src_off;
    uint16_t* dst = reinterpret_cast<uint16_t*>(arena + te.dst_off);
    const int c0 = cx * 64, k0 = ky * 64;
    #pragma unroll
    for (int v = threadIdx.x; v < 512; v += 256) {
        const int i = v >> 3, j = v & 7;
        const int k = k0 + i, c = c0 + j * 8;
        uint4 val = make_uint4(0, 0, 0, 0);
        if (k < te.K && c < te.C) val = *reinterpret_cast<const uint4*>(src + ((int64_t)k * te.RS + t) * te.C + c);
        uint2* d = reinterpret_cast<uint2*>(&tile[i * LD + j * 8]);
        d[0] = make_uint2(val.x, val.y);
        d[1] = make_uint2(val.z, val.w);
    }
    __syncthreads();
    #pragma unroll
    for (int v = threadIdx.x; v < 512; v += 256) {
        const int ci = v >> 3, kj = v & 7;
        const int c = c0 + ci, k = k0 + kj * 8;
        if (c < te.C && k < te.K) {
            uint32_t o[4];
            #pragma unroll
            for (int q = 0; q < 4; ++q)
                o[q] = (uint32_t)tile[(kj * 8 + 2 * q) * LD + ci] | ((uint32_t)tile[(kj * 8 + 2 * q + 1) * LD + ci] << 16);
            *reinterpret_cast<uint4*>(dst + ((int64_t)c * te.RS + t) * te.K + k) = make_uint4(o[0], o[1], o[2], o[3]);
        }
    }
}

void launch_weight_transpose_bf16(const uint16_t* w16, void* arena, const TransposeEntry* dev_table, int entries,
                                  int total_tiles, double bytes, hipStream_t st) {
    if (entries <= 0 || total_tiles <= 0) return;
    ProfScope ps("weight_transpose", 0.0, bytes, st);
    hipLaunchKernelGGL(weight_transpose_bf16_kernel, dim3(total_tiles), dim3(256), 0, st, w16, (unsigned char*)arena, dev_table, entries);
}

void launch_weight_transpose_all(int dtype, const float* w, void* arena, const TransposeEntry* dev_table, int entries,
                                 int total_tiles, double bytes, hipStream_t st) {
    if (entries <= 0 || total_tiles <= 0) return;
    ProfScope ps("weight_transpose", 0.0, bytes, st);
    if (dtype == 1)
        hipLaunchKernelGGL(weight_transpose_all_kernel<bf16_t>, dim3(total_tiles), dim3(256), 0, st, w, (unsigned char*)arena, dev_table, entries);
    else
        hipLaunchKernelGGL(weight_transpose_all_kernel<float>, dim3(total_tiles), dim3(256), 0, st, w, (unsigned char*)arena, dev_table, entries);
}

// ---------------------------------------------------------------------------
// out_x[i][:] = cast(data_x[idx[i]][:]) ; out_y[i] = data_y[idx[i]]
// grid: (chunks of the sample, n)
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void gather_kernel(const float* __restrict__ data_x, const int32_t* __restrict__ data_y,
                                                     const int64_t* __restrict__ idx, int64_t sample_elems,
                                                     T* __restrict__ out_x, int32_t* __restrict__ out_y) {
    const int i = blockIdx.y;
    const int64_t s = idx[i];
    const float* src = data_x + s * sample_elems;
    T* dst = out_x + (int64_t)i * sample_elems;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t t0 = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if ((sample_elems & 3) == 0) {
        for (int64_t q = t0; q < sample_elems / 4; q += stride) {
            const float4 f = reinterpret_cast<const float4*>(src)[q];
            dst[4 * q + 0] = Elem<T>::from_f32(f.x);
            dst[4 * q + 1] = Elem<T>::from_f32(f.y);
            dst[4 * q + 2] = Elem<T>::from_f32(f.z);
            dst[4 * q + 3] = Elem<T>::from_f32(f.w);
        }
    } else {
        for (int64_t q = t0; q < sample_elems; q += stride) dst[q] = Elem<T>::from_f32(src[q]);
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) out_y[i] = data_y[s];
}

// The same for images whose channel count is not a multiple of the vector
// width: every pixel is written as one 16-byte vector, padded with zeros, so
// that the first convolution can take the vector path.  grid: (pixel chunks, n)
template <typename T>
__global__ __launch_bounds__(256) void gather_pad_kernel(const float* __restrict__ data_x, const int32_t* __restrict__ data_y,
                                                         const int64_t* __restrict__ idx, int64_t pixels, int C,
                                                         T* __restrict__ out_x, int32_t* __restrict__ out_y) {
    constexpr int VEC = Elem<T>::VEC;
    const int i = blockIdx.y;
    const int64_t s = idx[i];
    const float* src = data_x + s * pixels * C;
    T* dst = out_x + (int64_t)i * pixels * VEC;
    for (int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; q < pixels; q += (int64_t)gridDim.x * blockDim.x) {
        Vec16<T> v;
        #pragma unroll
        for (int e = 0; e < VEC; ++e) v.e[e] = Elem<T>::from_f32(e < C ? src[q * C + e] : 0.f);
        store_vec(dst + q * VEC, v);
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) out_y[i] = data_y[s];
}

void launch_gather_pad(int dtype, const float* data_x, const int32_t* data_y, const int64_t* idx, int n, int64_t pixels,
                       int C, void* out_x, int32_t* out_y, hipStream_t st) {
    dim3 grid(grid_for(pixels, 256, 256), n);
    ProfScope ps("gather", 0.0, (4.0 * C + 16.0) * (double)pixels * n, st);
    if (dtype == 1)
        hipLaunchKernelGGL(gather_pad_kernel<bf16_t>, grid, dim3(256), 0, st, data_x, data_y, idx, pixels, C, (bf16_t*)out_x, out_y);
    else
        hipLaunchKernelGGL(gather_pad_kernel<float>, grid, dim3(256), 0, st, data_x, data_y, idx, pixels, C, (float*)out_x, out_y);
}

// dst[k][t][0..Cp) = cast(src[k][t][0..C)), zero beyond C  (weights of a convolution on padded images)
template <typename T>
__global__ __launch_bounds__(256) void pad_weights_kernel(const float* __restrict__ src, T* __restrict__ dst, int64_t rows, int C, int Cp) {
    const int64_t total = rows * Cp;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t r = i / Cp;
        const int c = (int)(i - r * Cp);
        dst[i] = Elem<T>::from_f32(c < C ? src[r * C + c] : 0.f);
    }
}

void launch_pad_weights(int dtype, const float* src, void* dst, int64_t rows, int C, int Cp, hipStream_t st) {
    const int grid = grid_for(rows * Cp, 256, 4096);
    ProfScope ps("pad_weights", 0.0, 4.0 * (double)rows * C + (dtype == 1 ? 2.0 : 4.0) * (double)rows * Cp, st);
    if (dtype == 1) hipLaunchKernelGGL(pad_weights_kernel<bf16_t>, dim3(grid), dim3(256), 0, st, src, (bf16_t*)dst, rows, C, Cp);
    else hipLaunchKernelGGL(pad_weights_kernel<float>, dim3(grid), dim3(256), 0, st, src, (float*)dst, rows, C, Cp);
}

// dst[r][0..C) = src[r][0..C) of rows of Cp floats (gradient of the padded weights back to the flat vector)
__global__ __launch_bounds__(256) void unpad_rows_kernel(const float* __restrict__ src, float* __restrict__ dst, int64_t rows, int C, int Cp) {
    const int64_t total = rows * C;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t r = i / C;
        dst[i] = src[r * Cp + (i - r * C)];
    }
}

void launch_unpad_rows(const float* src, float* dst, int64_t rows, int C, int Cp, hipStream_t st) {
    ProfScope ps("unpad_rows", 0.0, 8.0 * (double)rows * C, st);
    hipLaunchKernelGGL(unpad_rows_kernel, dim3(grid_for(rows * C, 256, 4096)), dim3(256), 0, st, src, dst, rows, C, Cp);
}

void launch_gather(int dtype, const float* data_x, const int32_t* data_y, const int64_t* idx, int n,
                   int64_t sample_elems, void* out_x, int32_t* out_y, hipStream_t st) {
    dim3 grid(grid_for(sample_elems / 4 + 1, 256, 64), n);
    ProfScope ps("gather", 0.0, (4.0 + (dtype == 1 ? 2.0 : 4.0)) * (double)sample_elems * n, st);
    if (dtype == 1)
        hipLaunchKernelGGL(gather_kernel<bf16_t>, grid, dim3(256), 0, st, data_x, data_y, idx, sample_elems,
                           (bf16_t*)out_x, out_y);
    else
        hipLaunchKernelGGL(gather_kernel<float>, grid, dim3(256), 0, st, data_x, data_y, idx, sample_elems,
                           (float*)out_x, out_y);
}

}  // namespace edl
