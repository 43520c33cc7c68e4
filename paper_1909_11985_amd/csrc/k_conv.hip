// Implicit-GEMM convolution on the matrix cores: forward, input gradient and
// weight gradient of a channels-last convolution (a fully connected layer is
// the 1x1 case on a 1x1 image).  These are the "computation-intensive
// kernels such as matrix multiplication" of the paper's section 2.1.
//
// All three are Out[M][Nn] = sum_kk A[m][kk] * B[j][kk] with different gathers:
//
//   forward   M = N*Ho*Wo pixels   Nn = K      kk = (r,s,c)   A = x gathered, B = w[K][R][S][C]
//   dgrad     M = N*H*W   pixels   Nn = C      kk = (r,s,k)   A = dy gathered, B = wT[C][R][S][K]
//   wgrad     M = K               Nn = R*S*C   kk = pixel     A = dy^T, B = x^T gathered
//
// A workgroup of 4 waves owns a BM x BN output tile and walks the reduction in
// steps of BK = 32 elements.  Tiles are staged in LDS with the reduction index
// innermost (rows padded by one 16-byte vector, which makes the 16-byte
// fragment reads conflict-free); each wave then feeds 32x32 MFMA tiles from
// 16-byte fragments: one v_mfma_f32_32x32x16_bf16 per fragment pair for bf16,
// four v_mfma_f32_32x32x2_f32 for float32 (lane L of a fragment holds row L%32
// and the reduction slice selected by L/32; both operands use the same slice
// order, so any order is a valid contraction).  Global loads of the next tile
// are issued before the MFMAs of the current one.  For the weight gradient the
// reduction index (the pixel) is the slow index in memory, so its tiles are
// transposed on the way into LDS; its reduction is cut into splits whose
// float32 partial tiles are added by a second kernel in split order.
#include "dev_common.h"
#include "kernels.h"
#include "profiler.h"

namespace edl {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

struct ConvArgs {
    const void* A;
    const void* B;
    void* out;
    const float* bias;
    int N, H, W, C, K, R, S, stride, pad, Ho, Wo;
    int M, Nn, Kred;
    int relu, out_fp32, accumulate;
    int vecA, vecB;
    int ksplit;  // reduction elements per blockIdx.z
};

template <typename T> struct Frag;
template <> struct Frag<bf16_t> {
    static __device__ __forceinline__ void mma(const uint4& a, const uint4& b, floatx16& c) {
        c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
};
template <> struct Frag<float> {
    static __device__ __forceinline__ void mma(const uint4& a, const uint4& b, floatx16& c) {
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), c, 0, 0, 0);
    }
};

// context of one tile row for the pixel-indexed operand of forward / dgrad
struct RowCtx {
    int64_t base;
    int h0, w0;
    bool valid;
};

template <typename T, int MODE>
__device__ __forceinline__ RowCtx make_row(const ConvArgs& a, int m) {
    RowCtx c;
    c.valid = m < a.M;
    if (MODE == CONV_FWD) {
        const int hw = a.Ho * a.Wo;
        const int n = m / hw, rem = m - n * hw;
        const int ho = rem / a.Wo, wo = rem - ho * a.Wo;
        c.h0 = ho * a.stride - a.pad;
        c.w0 = wo * a.stride - a.pad;
        c.base = (((int64_t)n * a.H + c.h0) * a.W + c.w0) * a.C;
    } else {
        const int hw = a.H * a.W;
        const int n = m / hw, rem = m - n * hw;
        const int h = rem / a.W, w = rem - h * a.W;
        c.h0 = h + a.pad;
        c.w0 = w + a.pad;
        c.base = (int64_t)n * a.Ho * a.Wo * a.K;
    }
    return c;
}

// element offset of A[m][kk] for forward / dgrad; ok = inside the image
template <int MODE>
__device__ __forceinline__ int64_t a_offset(const ConvArgs& a, const RowCtx& c, int kk, bool& ok) {
    if (MODE == CONV_FWD) {
        const int tap = kk / a.C, ch = kk - tap * a.C;
        const int r = tap / a.S, s = tap - r * a.S;
        const int h = c.h0 + r, w = c.w0 + s;
        ok = c.valid && kk < a.Kred && (unsigned)h < (unsigned)a.H && (unsigned)w < (unsigned)a.W;
        return c.base + ((int64_t)r * a.W + s) * a.C + ch;
    } else {
        const int tap = kk / a.K, k = kk - tap * a.K;
        const int r = tap / a.S, s = tap - r * a.S;
        const int hn = c.h0 - r, wn = c.w0 - s;
        int ho = hn, wo = wn;
        bool on_grid = true;
        if (a.stride != 1) {
            ho = hn / a.stride;
            wo = wn / a.stride;
            on_grid = (ho * a.stride == hn) && (wo * a.stride == wn);
        }
        ok = c.valid && kk < a.Kred && hn >= 0 && wn >= 0 && on_grid && ho < a.Ho && wo < a.Wo;
        return c.base + ((int64_t)ho * a.Wo + wo) * a.K + k;
    }
}

template <typename T, int MODE, int WM, int WN, int TM, int TN>
__global__ __launch_bounds__(256) void conv_igemm_kernel(ConvArgs a) {
    constexpr int BM = WM * TM * 32, BN = WN * TN * 32, BK = 32;
    constexpr int VEC = Elem<T>::VEC;
    constexpr int LDK = BK + VEC;
    constexpr int KV = BK / VEC;                 // vectors per tile row (reduction innermost)
    constexpr int ITER_A = (MODE == CONV_WGRAD) ? (BK * (BM / VEC) + 255) / 256 : (BM * KV + 255) / 256;
    constexpr int ITER_B = (MODE == CONV_WGRAD) ? (BK * (BN / VEC) + 255) / 256 : (BN * KV + 255) / 256;
    static_assert(WM * WN == 4, "four waves per workgroup");

    __shared__ __attribute__((aligned(16))) T As[BM * LDK];
    __shared__ __attribute__((aligned(16))) T Bs[BN * LDK];

    const T* __restrict__ Ag = (const T*)a.A;
    const T* __restrict__ Bg = (const T*)a.B;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int m0 = blockIdx.x * BM, n0 = blockIdx.y * BN;
    const int kbeg = blockIdx.z * a.ksplit;
    int kend = kbeg + a.ksplit;
    if (kend > a.Kred) kend = a.Kred;
    const int nk = (kend - kbeg + BK - 1) / BK;

    Vec16<T> ra[ITER_A], rb[ITER_B];

    // ---- per-thread constants of the gathers --------------------------------
    RowCtx rowA[ITER_A];
    int wg_r = 0, wg_s = 0, wg_c = 0;  // wgrad: tap and channel of this thread's B rows
    if (MODE != CONV_WGRAD) {
        #pragma unroll
        for (int it = 0; it < ITER_A; ++it) {
            const int v = tid + it * 256;
            rowA[it] = make_row<T, MODE>(a, m0 + v / KV);
        }
    } else {
        constexpr int RVB = BN / VEC;
        const int j0 = n0 + (tid % RVB) * VEC;
        const int tap = j0 / a.C;
        wg_c = j0 - tap * a.C;
        wg_r = tap / a.S;
        wg_s = tap - wg_r * a.S;
    }

    auto load_tiles = [&](int k0) {
        if (MODE != CONV_WGRAD) {
            // A: pixel rows, reduction innermost
            #pragma unroll
            for (int it = 0; it < ITER_A; ++it) {
                const int v = tid + it * 256;
                const int kk0 = k0 + (v % KV) * VEC;
                ra[it].u = make_uint4(0, 0, 0, 0);
                if (BM * KV % 256 != 0 && v >= BM * KV) continue;
                if (a.vecA) {
                    bool ok;
                    const int64_t off = a_offset<MODE>(a, rowA[it], kk0, ok);
                    if (ok && kk0 < kend) ra[it] = load_vec(Ag + off);
                } else {
                    #pragma unroll
                    for (int e = 0; e < VEC; ++e) {
                        bool ok;
                        const int64_t off = a_offset<MODE>(a, rowA[it], kk0 + e, ok);
                        if (ok && kk0 + e < kend) ra[it].e[e] = Ag[off];
                    }
                }
            }
            // B: weight rows, contiguous in the reduction index
            #pragma unroll
            for (int it = 0; it < ITER_B; ++it) {
                const int v = tid + it * 256;
                const int kk0 = k0 + (v % KV) * VEC;
                const int j = n0 + v / KV;
                rb[it].u = make_uint4(0, 0, 0, 0);
                if (BN * KV % 256 != 0 && v >= BN * KV) continue;
                if (j < a.Nn) {
                    const int64_t off = (int64_t)j * a.Kred + kk0;
                    if (a.vecB) {
                        if (kk0 < kend) rb[it] = load_vec(Bg + off);
                    } else {
                        #pragma unroll
                        for (int e = 0; e < VEC; ++e)
                            if (kk0 + e < kend) rb[it].e[e] = Bg[off + e];
                    }
                }
            }
        } else {
            // A = dy[pixel][k]: vectors along k for one pixel
            constexpr int RVA = BM / VEC;
            #pragma unroll
            for (int it = 0; it < ITER_A; ++it) {
                const int v = tid + it * 256;
                const int row0 = m0 + (v % RVA) * VEC;
                const int mm = k0 + v / RVA;
                ra[it].u = make_uint4(0, 0, 0, 0);
                if (BK * RVA % 256 != 0 && v >= BK * RVA) continue;
                if (mm < kend) {
                    const int64_t off = (int64_t)mm * a.K + row0;
                    if (a.vecA) {
                        if (row0 < a.M) ra[it] = load_vec(Ag + off);
                    } else {
                        #pragma unroll
                        for (int e = 0; e < VEC; ++e)
                            if (row0 + e < a.M) ra[it].e[e] = Ag[off + e];
                    }
                }
            }
            // B = x gathered at (pixel, tap): vectors along c
            constexpr int RVB = BN / VEC;
            const int hw = a.Ho * a.Wo;
            #pragma unroll
            for (int it = 0; it < ITER_B; ++it) {
                const int v = tid + it * 256;
                const int mm = k0 + v / RVB;
                rb[it].u = make_uint4(0, 0, 0, 0);
                if (BK * RVB % 256 != 0 && v >= BK * RVB) continue;
                if (mm < kend) {
                    const int n = mm / hw, rem = mm - n * hw;
                    const int ho = rem / a.Wo, wo = rem - ho * a.Wo;
                    const int hb = ho * a.stride - a.pad, wb = wo * a.stride - a.pad;
                    if (a.vecB) {
                        const int j0 = n0 + (v % RVB) * VEC;
                        const int h = hb + wg_r, w = wb + wg_s;
                        if (j0 < a.Nn && (unsigned)h < (unsigned)a.H && (unsigned)w < (unsigned)a.W)
                            rb[it] = load_vec(Bg + (((int64_t)n * a.H + h) * a.W + w) * a.C + wg_c);
                    } else {
                        #pragma unroll
                        for (int e = 0; e < VEC; ++e) {
                            const int j = n0 + (v % RVB) * VEC + e;
                            const int tap = j / a.C, ch = j - tap * a.C;
                            const int r = tap / a.S, s = tap - r * a.S;
                            const int h = hb + r, w = wb + s;
                            if (j < a.Nn && (unsigned)h < (unsigned)a.H && (unsigned)w < (unsigned)a.W)
                                rb[it].e[e] = Bg[(((int64_t)n * a.H + h) * a.W + w) * a.C + ch];
                        }
                    }
                }
            }
        }
    };

    auto store_tiles = [&]() {
        if (MODE != CONV_WGRAD) {
            #pragma unroll
            for (int it = 0; it < ITER_A; ++it) {
                const int v = tid + it * 256;
                if (BM * KV % 256 != 0 && v >= BM * KV) continue;
                store_vec(&As[(v / KV) * LDK + (v % KV) * VEC], ra[it]);
            }
            #pragma unroll
            for (int it = 0; it < ITER_B; ++it) {
                const int v = tid + it * 256;
                if (BN * KV % 256 != 0 && v >= BN * KV) continue;
                store_vec(&Bs[(v / KV) * LDK + (v % KV) * VEC], rb[it]);
            }
        } else {
            constexpr int RVA = BM / VEC, RVB = BN / VEC;
            #pragma unroll
            for (int it = 0; it < ITER_A; ++it) {
                const int v = tid + it * 256;
                if (BK * RVA % 256 != 0 && v >= BK * RVA) continue;
                #pragma unroll
                for (int e = 0; e < VEC; ++e) As[((v % RVA) * VEC + e) * LDK + v / RVA] = ra[it].e[e];
            }
            #pragma unroll
            for (int it = 0; it < ITER_B; ++it) {
                const int v = tid + it * 256;
                if (BK * RVB % 256 != 0 && v >= BK * RVB) continue;
                #pragma unroll
                for (int e = 0; e < VEC; ++e) Bs[((v % RVB) * VEC + e) * LDK + v / RVB] = rb[it].e[e];
            }
        }
    };

    floatx16 acc[TM][TN];
    #pragma unroll
    for (int i = 0; i < TM; ++i)
        #pragma unroll
        for (int j = 0; j < TN; ++j)
            #pragma unroll
            for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.f;

    if (nk > 0) load_tiles(kbeg);
    for (int kt = 0; kt < nk; ++kt) {
        store_tiles();
        __syncthreads();
        if (kt + 1 < nk) load_tiles(kbeg + (kt + 1) * BK);
        constexpr int KG = 2 * VEC;  // reduction elements one fragment pair covers
        #pragma unroll
        for (int g = 0; g < BK / KG; ++g) {
            uint4 fa[TM], fb[TN];
            #pragma unroll
            for (int i = 0; i < TM; ++i)
                fa[i] = *reinterpret_cast<const uint4*>(&As[((wm * TM + i) * 32 + (lane & 31)) * LDK + g * KG + (lane >> 5) * VEC]);
            #pragma unroll
            for (int j = 0; j < TN; ++j)
                fb[j] = *reinterpret_cast<const uint4*>(&Bs[((wn * TN + j) * 32 + (lane & 31)) * LDK + g * KG + (lane >> 5) * VEC]);
            #pragma unroll
            for (int i = 0; i < TM; ++i)
                #pragma unroll
                for (int j = 0; j < TN; ++j) Frag<T>::mma(fa[i], fb[j], acc[i][j]);
        }
        __syncthreads();
    }

    // ---- epilogue: lane holds column lane%32, rows (q/4)*8 + (lane/32)*4 + q%4 ----
    #pragma unroll
    for (int i = 0; i < TM; ++i) {
        #pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = n0 + (wn * TN + j) * 32 + (lane & 31);
            if (col >= a.Nn) continue;
            const float bias = (MODE == CONV_FWD && a.bias) ? a.bias[col] : 0.f;
            #pragma unroll
            for (int q = 0; q < 16; ++q) {
                const int row = m0 + (wm * TM + i) * 32 + (q >> 2) * 8 + (lane >> 5) * 4 + (q & 3);
                if (row >= a.M) continue;
                float v = acc[i][j][q];
                if (MODE == CONV_FWD) {
                    v += bias;
                    if (a.relu) v = v > 0.f ? v : 0.f;
                    const int64_t o = (int64_t)row * a.Nn + col;
                    if (a.out_fp32) ((float*)a.out)[o] = v;
                    else ((T*)a.out)[o] = Elem<T>::from_f32(v);
                } else if (MODE == CONV_DGRAD) {
                    const int64_t o = (int64_t)row * a.Nn + col;
                    T* dst = (T*)a.out;
                    if (a.accumulate) v += Elem<T>::to_f32(dst[o]);
                    dst[o] = Elem<T>::from_f32(v);
                } else {
                    ((float*)a.out)[((int64_t)blockIdx.z * a.M + row) * a.Nn + col] = v;
                }
            }
        }
    }
}

// dw[i] = sum over splits, in split order
__global__ __launch_bounds__(256) void wgrad_reduce_kernel(const float* __restrict__ part, float* __restrict__ dw, int64_t n,
                                                           int splits) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        float s = part[i];
        for (int k = 1; k < splits; ++k) s += part[(int64_t)k * n + i];
        dw[i] = s;
    }
}

// ---------------------------------------------------------------------------
// host side: tile selection and launch
// ---------------------------------------------------------------------------
enum TileCfg { T128x128, T128x64, T128x32, T64x64 };

static TileCfg pick_tile(int M, int Nn, int* bm, int* bn) {
    TileCfg t;
    if (Nn <= 32) t = T128x32;
    else if (Nn <= 64) t = (M >= 128) ? T128x64 : T64x64;
    else {
        const int64_t tiles = (int64_t)((M + 127) / 128) * ((Nn + 127) / 128);
        t = (tiles >= 256 && M >= 128) ? T128x128 : T64x64;
    }
    switch (t) {
        case T128x128: *bm = 128; *bn = 128; break;
        case T128x64: *bm = 128; *bn = 64; break;
        case T128x32: *bm = 128; *bn = 32; break;
        default: *bm = 64; *bn = 64; break;
    }
    return t;
}

template <typename T, int MODE>
static void launch_cfg(TileCfg t, dim3 grid, const ConvArgs& a, hipStream_t st) {
    switch (t) {
        case T128x128: hipLaunchKernelGGL((conv_igemm_kernel<T, MODE, 2, 2, 2, 2>), grid, dim3(256), 0, st, a); break;
        case T128x64: hipLaunchKernelGGL((conv_igemm_kernel<T, MODE, 2, 2, 2, 1>), grid, dim3(256), 0, st, a); break;
        case T128x32: hipLaunchKernelGGL((conv_igemm_kernel<T, MODE, 4, 1, 1, 1>), grid, dim3(256), 0, st, a); break;
        default: hipLaunchKernelGGL((conv_igemm_kernel<T, MODE, 2, 2, 1, 1>), grid, dim3(256), 0, st, a); break;
    }
}

static const char* conv_label(int dtype, int mode, TileCfg t) {
    static const char* names[2][3][4] = {
        {{"conv_fwd_f32_128x128", "conv_fwd_f32_128x64", "conv_fwd_f32_128x32", "conv_fwd_f32_64x64"},
         {"conv_dgrad_f32_128x128", "conv_dgrad_f32_128x64", "conv_dgrad_f32_128x32", "conv_dgrad_f32_64x64"},
         {"conv_wgrad_f32_128x128", "conv_wgrad_f32_128x64", "conv_wgrad_f32_128x32", "conv_wgrad_f32_64x64"}},
        {{"conv_fwd_bf16_128x128", "conv_fwd_bf16_128x64", "conv_fwd_bf16_128x32", "conv_fwd_bf16_64x64"},
         {"conv_dgrad_bf16_128x128", "conv_dgrad_bf16_128x64", "conv_dgrad_bf16_128x32", "conv_dgrad_bf16_64x64"},
         {"conv_wgrad_bf16_128x128", "conv_wgrad_bf16_128x64", "conv_wgrad_bf16_128x32", "conv_wgrad_bf16_64x64"}}};
    return names[dtype == 1 ? 1 : 0][mode][(int)t];
}

template <int MODE>
static void launch_mode(int dtype, TileCfg t, dim3 grid, const ConvArgs& a, hipStream_t st) {
    // algorithmic work: 2*M*N*K flops; operands and result touched once
    const double esz = dtype == 1 ? 2.0 : 4.0;
    const double flops = 2.0 * (double)a.M * a.Nn * a.Kred;
    double bytes;
    if (MODE == CONV_FWD) bytes = esz * ((double)a.N * a.H * a.W * a.C + (double)a.Nn * a.Kred) + (a.out_fp32 ? 4.0 : esz) * (double)a.M * a.Nn;
    else if (MODE == CONV_DGRAD) bytes = esz * ((double)a.N * a.Ho * a.Wo * a.K + (double)a.Nn * a.Kred + (double)a.M * a.Nn);
    else bytes = esz * ((double)a.Kred * a.K + (double)a.N * a.H * a.W * a.C) + 4.0 * (double)a.M * a.Nn;
    ProfScope ps(conv_label(dtype, MODE, t), flops, bytes, st);
    if (dtype == 1) launch_cfg<bf16_t, MODE>(t, grid, a, st);
    else launch_cfg<float, MODE>(t, grid, a, st);
}

static ConvArgs base_args(const ConvGeom& g) {
    ConvArgs a = {};
    a.N = g.N; a.H = g.H; a.W = g.W; a.C = g.C; a.K = g.K; a.R = g.R; a.S = g.S;
    a.stride = g.stride; a.pad = g.pad; a.Ho = g.Ho; a.Wo = g.Wo;
    return a;
}

void launch_conv_fwd(int dtype, const ConvGeom& g, const void* x, const void* w, const float* bias, bool relu,
                     bool out_fp32, void* y, hipStream_t st) {
    const int VEC = dtype == 1 ? 8 : 4;
    ConvArgs a = base_args(g);
    a.A = x; a.B = w; a.out = y; a.bias = bias;
    a.M = g.N * g.Ho * g.Wo; a.Nn = g.K; a.Kred = g.R * g.S * g.C;
    a.relu = relu; a.out_fp32 = out_fp32;
    a.vecA = (g.C % VEC == 0); a.vecB = (a.Kred % VEC == 0);
    a.ksplit = a.Kred;
    int bm, bn;
    const TileCfg t = pick_tile(a.M, a.Nn, &bm, &bn);
    launch_mode<CONV_FWD>(dtype, t, dim3((a.M + bm - 1) / bm, (a.Nn + bn - 1) / bn, 1), a, st);
}

void launch_conv_dgrad(int dtype, const ConvGeom& g, const void* dy, const void* wT, bool accumulate, void* dx,
                       hipStream_t st) {
    const int VEC = dtype == 1 ? 8 : 4;
    ConvArgs a = base_args(g);
    a.A = dy; a.B = wT; a.out = dx;
    a.M = g.N * g.H * g.W; a.Nn = g.C; a.Kred = g.R * g.S * g.K;
    a.accumulate = accumulate;
    a.vecA = (g.K % VEC == 0); a.vecB = (a.Kred % VEC == 0);
    a.ksplit = a.Kred;
    int bm, bn;
    const TileCfg t = pick_tile(a.M, a.Nn, &bm, &bn);
    launch_mode<CONV_DGRAD>(dtype, t, dim3((a.M + bm - 1) / bm, (a.Nn + bn - 1) / bn, 1), a, st);
}

struct WgradPlan {
    TileCfg t;
    int bm, bn, splits, ksplit;
    int64_t tiles;
};

static WgradPlan plan_wgrad(const ConvGeom& g) {
    WgradPlan p;
    const int M = g.K, Nn = g.R * g.S * g.C, Kred = g.N * g.Ho * g.Wo;
    // tile choice by shape only (the split supplies the parallelism)
    if (Nn <= 32) p.t = T128x32;
    else if (M <= 64 || Nn <= 64) p.t = (Nn <= 64 && M >= 128) ? T128x64 : T64x64;
    else p.t = T128x128;
    switch (p.t) {
        case T128x128: p.bm = 128; p.bn = 128; break;
        case T128x64: p.bm = 128; p.bn = 64; break;
        case T128x32: p.bm = 128; p.bn = 32; break;
        default: p.bm = 64; p.bn = 64; break;
    }
    p.tiles = (int64_t)((M + p.bm - 1) / p.bm) * ((Nn + p.bn - 1) / p.bn);
    int64_t splits = (1024 + p.tiles - 1) / p.tiles;
    const int64_t max_splits = (Kred + 127) / 128;  // at least 4 reduction steps per split
    if (splits > max_splits) splits = max_splits;
    if (splits < 1) splits = 1;
    int64_t ks = (Kred + splits - 1) / splits;
    ks = (ks + 31) / 32 * 32;
    p.ksplit = (int)ks;
    p.splits = (int)((Kred + ks - 1) / ks);
    return p;
}

size_t conv_wgrad_scratch_bytes(const ConvGeom& g) {
    const WgradPlan p = plan_wgrad(g);
    if (p.splits <= 1) return 0;
    return (size_t)p.splits * g.K * g.R * g.S * g.C * sizeof(float);
}

void launch_conv_wgrad(int dtype, const ConvGeom& g, const void* x, const void* dy, float* dw, float* scratch,
                       size_t scratch_bytes, hipStream_t st) {
    const int VEC = dtype == 1 ? 8 : 4;
    const WgradPlan p = plan_wgrad(g);
    ConvArgs a = base_args(g);
    a.A = dy; a.B = x;
    a.M = g.K; a.Nn = g.R * g.S * g.C; a.Kred = g.N * g.Ho * g.Wo;
    a.vecA = (g.K % VEC == 0); a.vecB = (g.C % VEC == 0);
    a.ksplit = p.ksplit;
    const int64_t n = (int64_t)a.M * a.Nn;
    const bool direct = p.splits <= 1 || scratch == nullptr || scratch_bytes < (size_t)p.splits * n * sizeof(float);
    if (direct) {
        a.ksplit = a.Kred;
        a.out = dw;
    } else {
        a.out = scratch;
    }
    const dim3 grid((a.M + p.bm - 1) / p.bm, (a.Nn + p.bn - 1) / p.bn, direct ? 1 : p.splits);
    launch_mode<CONV_WGRAD>(dtype, p.t, grid, a, st);
    if (!direct) {
        int64_t blocks = (n + 255) / 256;
        if (blocks > 4096) blocks = 4096;
        ProfScope ps("wgrad_reduce", 0.0, 4.0 * (double)n * (p.splits + 1), st);
        hipLaunchKernelGGL(wgrad_reduce_kernel, dim3((int)blocks), dim3(256), 0, st, scratch, dw, n, p.splits);
    }
}

}  // namespace edl
