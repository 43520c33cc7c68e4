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
// tiles of BK elements (eight 16-byte vectors per row).  Each wave feeds 32x32
// MFMA tiles from 16-byte fragments: one v_mfma_f32_32x32x16_bf16 per fragment
// pair for bf16, four v_mfma_f32_32x32x2_f32 for float32 (lane L of a fragment
// holds row L%32 and the reduction slice selected by L/32; both operands use
// the same slice order, so any order is a valid contraction).
//
//  * loads: 16-byte buffer loads whose range check returns zeros, so padding
//    taps, ragged edges and the reduction tail need no branch.  The vector
//    kernel (FAST) sends them straight into LDS (buffer_load ... lds: lane L's
//    16 bytes land at M0 + 16*L), PF+1 LDS stages deep, with explicit vmcnt
//    waits and one barrier per tile; it has no element-wise path.  The float32
//    weight gradient, and a second, slow instantiation for operands that are
//    not vector-shaped, keep the register-staged path: their loads land in
//    registers while the previous tile is contracted, then go to the other of
//    two LDS stages.
//  * forward / dgrad tiles: rows of BK elements; on the direct path unpadded,
//    the 16-byte chunks of a row XOR-swizzled by the row index, otherwise padded
//    by one vector (conflict-free fragment reads either way).  Weight-gradient
//    tiles: the reduction index (the pixel) is the slow index in memory; bf16
//    tiles stay [pixel][channel] and are transposed on the way out of LDS
//    (ds_read_tr16_b64), float32 tiles are 32-bit words read one by one.
//  * dgrad of a strided convolution runs once per residue class of the input
//    pixel modulo the stride and contracts only the taps that reach the class.
//  * epilogue: through LDS as float32, out as 16-byte vectors (bf16 packed by
//    the hardware conversion).
//  * long reductions of small problems, and every weight gradient, are cut
//    across workgroups; the float32 partial tiles are summed in split order by
//    a second kernel (no float atomics: results are bit-reproducible).
#include <algorithm>
#include <deque>
#include <string>

#include "dev_common.h"
#include "kernels.h"
#include "profiler.h"
#include "tune.h"

// 1: LDS fragment reads run one fragment group ahead of the MFMAs (tiles of more than one MFMA per group;
// measured -6% on the 128x128 weight gradient, nothing on the others)
#ifndef EDL_FRAG_AHEAD
#define EDL_FRAG_AHEAD 1
#endif

// 1: the vector kernels of forward / dgrad load their tiles from global memory straight into LDS
// (16 bytes per lane, no register staging, PF + 1 LDS stages); 0: through registers, two stages
#ifndef EDL_DIRECT_LDS
#define EDL_DIRECT_LDS 1
#endif
// the same for the bf16 weight gradient
#ifndef EDL_DIRECT_WG
#define EDL_DIRECT_WG 1
#endif

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
    unsigned bytesA, bytesB;  // extents of the two operands (for the range-checked vector loads)
    // dgrad of a strided convolution, one launch per residue class of the input
    // pixel (h % stride, w % stride) = (ph, pw): only the taps r = r0, r0+stride, ...
    // (nr of them) and s = s0, ... (ns) reach such a pixel, so the reduction runs
    // over nr*ns*K instead of R*S*K.  Hc x Wc pixels per image are in the class.
    // For stride 1 (and the other modes): ph = pw = r0 = s0 = 0, nr = R, ns = S.
    int ph, pw, Hc, Wc, r0, s0, nr, ns;
    int ldb;     // fwd/dgrad: elements between consecutive rows of B
    float* partial;  // fwd/dgrad with a cut reduction: float32 [split][M][Nn] partial sums, else null
    // dgrad with accumulate: the gradient that is added to is read here (same shape and layout as the output;
    // null: from the output buffer itself).  Lets the first reader of a residual join take the shortcut's part
    // from where it already lies instead of from a copy.
    const void* acc_src;
    // fwd, vector path, whole reduction: if not null, the column sums of the stored output and of its
    // squares over this tile's rows go to stats[c * kRedRowBlocks + row tile] and
    // stats[(Nn + c) * kRedRowBlocks + row tile] (the layout of the batch-norm reduction's partial sums)
    float* stats;
    // dgrad, vector path, whole reduction, stride 1, not accumulating: the layer that produced this
    // convolution's input ends in a ReLU, and its backward starts with "gradient times (activation > 0)"
    // followed by per-channel sums of that.  With mask_act (the activation, same shape as the output) the
    // gradient is stored already masked, and its column sums over the tile's rows go to msum (the layout of
    // stats above): kind 0 = sum of the masked gradient; kind 1 = sum of masked gradient * (xin - mean) * rstd
    // if xin (the producing batch norm's input) and mean_rstd ([mean[Nn], rstd[Nn]]) are given, else unused.
    const void* mask_act;
    const void* xin;
    const float* mean_rstd;
    float* msum;
    // ceil(2^40 / d) for d = channels per tap and d = taps per kernel row: n / d == (n * magic) >> 40
    // for n * d < 2^40, which keeps the tap bookkeeping of the load loop free of branches
    unsigned long long magic_inner, magic_taps;
    // the same for d = pixels per image and d = pixels per image row of the row index's pixel grid
    // (output pixels in the forward pass, the residue class's input pixels in dgrad), and for the tile grid
    unsigned long long magic_hw, magic_w, magic_gx, magic_gy;
    int stride_shift;                  // dgrad vector path: log2 of the stride (a power of two there)
    int red_stride;                    // floats between the partial column sums of consecutive channels
    // Tile grid (gx row tiles, gy column tiles, gz cuts of the reduction), launched
    // as gx*gy*gz workgroups in one dimension.  The hardware hands consecutive
    // workgroups to the eight dies in turn and each die has its own L2, so with
    // xcd_chunked the kernel gives every die one contiguous run of the tile
    // sequence; n_fastest chooses which operand the neighbours of a run share.
    int gx, gy, gz, xcd_chunked, n_fastest;
};

__device__ __forceinline__ int fast_div(int n, unsigned long long magic) {
    return (int)(((unsigned long long)(unsigned)n * magic) >> 40);
}

// (row tile, column tile, reduction cut) of this workgroup
__device__ __forceinline__ void tile_of_block(const ConvArgs& a, int& bx, int& by, int& bz) {
    const int total = a.gx * a.gy * a.gz;
    int l = blockIdx.x;
    if (a.xcd_chunked) {
        const int q = total >> 3, r = total & 7, die = l & 7, slot = l >> 3;
        l = die * q + (die < r ? die : r) + slot;   // die d owns q (+1 for d < r) consecutive tiles
    }
    const bool mg = a.magic_gx != 0;   // 0: the grid is too large for the multiply-shift division
    if (a.n_fastest) {
        const int t = mg ? fast_div(l, a.magic_gy) : l / a.gy;
        by = l - t * a.gy;
        bz = mg ? fast_div(t, a.magic_gx) : t / a.gx;
        bx = t - bz * a.gx;
    } else {
        const int t = mg ? fast_div(l, a.magic_gx) : l / a.gx;
        bx = l - t * a.gx;
        bz = mg ? fast_div(t, a.magic_gy) : t / a.gy;
        by = t - bz * a.gy;
    }
}


// 16-byte load through a buffer descriptor: an offset at or beyond the
// descriptor's extent returns zeros, so padding taps, ragged tile edges and
// the tail of the reduction need no branch and every load of a tile can be in
// flight at once.
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
constexpr unsigned kOutOfRange = 0x80000000u;   // operands are smaller than 2 GiB (checked by the launchers)

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, unsigned bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, bytes, 0x00020000);
}
// The same load, landing in LDS instead of registers: lane L's 16 bytes go to LDS byte address
// lds_wave_base + 16*L (lds_wave_base is wave-uniform and travels in M0); a lane whose offset is out of range
// writes zeros.  The instruction is issued from inline assembly, so the compiler does not know of the
// outstanding LDS write: the caller orders it against LDS reads with wait_vmcnt<> and a barrier, and no other
// code of the kernel may use M0.
typedef int i32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ i32x4 make_rsrc_words(const void* p, unsigned bytes) {
    const uint64_t a = (uint64_t)p;
    const i32x4 r = {(int)(uint32_t)a, (int)((uint32_t)(a >> 32) & 0xffffu), (int)bytes, 0x00020000};
    return r;
}
__device__ __forceinline__ void buffer_load16_to_lds(i32x4 rsrc, unsigned lds_wave_base, unsigned byte_offset) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :: "s"(lds_wave_base), "v"(byte_offset), "s"(rsrc) : "memory");
}
// waits until at most N of this wave's vector-memory loads are outstanding (they complete in order)
template <int N> __device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

__device__ __forceinline__ uint4 buffer_load16(__amdgpu_buffer_rsrc_t r, unsigned byte_offset) {
    const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, byte_offset, 0, 0);
    return make_uint4(v.x, v.y, v.z, v.w);
}

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

// bf16 wgrad tiles in LDS: row = pixel of the reduction step, WIDTH channels per row, no padding; the
// 16-channel (32-byte) chunks of a row are permuted by the row's low bits.  A transposing read (tr_frag) takes,
// per 32 lanes, two neighbouring chunks of four consecutive pixel rows; those eight 32-byte pieces must fall
// into the eight different 32-byte bank groups.  Rows of 256 bytes (WIDTH 128) all start at the same bank, so
// the row moves its chunk pair by two chunks per row (XOR with 2 * (pixel % 4); XOR with pixel % 4, as the
// narrower tiles use, would put the pairs of rows 0/1 and 2/3 on top of each other: measured as 11% of the
// kernel's time in LDS bank conflicts).  Rows of 128 and 64 bytes are already spread by their own offsets.
template <int WIDTH>
__device__ __forceinline__ int wg_swizzle(int pixel) {
    return WIDTH >= 128 ? ((pixel & 3) << 1) : WIDTH >= 64 ? (pixel & 3) : (pixel & (WIDTH / 16 - 1));
}
template <int WIDTH>
__device__ __forceinline__ int wg_lds_index(int pixel, int ch) {
    return pixel * WIDTH + ((((ch >> 4) ^ wg_swizzle<WIDTH>(pixel)) << 4) | (ch & 15));
}

// MFMA operand of a 32-channel tile for reduction pixels [p16 + 8*(lane/32), +8) from such an LDS tile.
// ds_read_tr16_b64 hands lane l of a 16-lane group element (l % 4) of the four 16-bit values read by
// lanes l/4, l/4 + 4, l/4 + 8, l/4 + 12 of the group (lane layout measured on gfx950).  With lane s
// reading pixel s/4, channels 4*(s%4)..+3 of a 16-channel chunk, lane l therefore receives channel l of
// the chunk for four consecutive pixels; two reads give the operand's eight.
typedef short shortx4 __attribute__((ext_vector_type(4)));
template <int WIDTH>
__device__ __forceinline__ uint4 tr_frag(const bf16_t* tile, int ch32, int p16, int lane) {
    const int ch = ch32 + ((lane >> 4) & 1) * 16 + 4 * (lane & 3);
    const int p0 = p16 + (lane >> 5) * 8 + ((lane & 15) >> 2);
    typedef shortx4 __attribute__((address_space(3))) * lds_ptr;
    const shortx4 r0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(tile + wg_lds_index<WIDTH>(p0, ch)));
    const shortx4 r1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(tile + wg_lds_index<WIDTH>(p0 + 4, ch)));
    const uint2 a = __builtin_bit_cast(uint2, r0), b = __builtin_bit_cast(uint2, r1);
    return make_uint4(a.x, a.y, b.x, b.y);
}

// context of one tile row for the pixel-indexed operand of forward / dgrad
struct RowCtx {
    int64_t base;
    int h0, w0;
    bool valid;
};

template <int MODE, bool FAST>
__device__ __forceinline__ RowCtx make_row(const ConvArgs& a, int m) {
    RowCtx c;
    c.valid = m < a.M;
    if (MODE == CONV_FWD) {
        const int hw = a.Ho * a.Wo;
        const int n = FAST ? fast_div(m, a.magic_hw) : m / hw, rem = m - n * hw;
        const int ho = FAST ? fast_div(rem, a.magic_w) : rem / a.Wo, wo = rem - ho * a.Wo;
        c.h0 = ho * a.stride - a.pad;
        c.w0 = wo * a.stride - a.pad;
        c.base = (((int64_t)n * a.H + c.h0) * a.W + c.w0) * a.C;
    } else {
        const int hw = a.Hc * a.Wc;
        const int n = FAST ? fast_div(m, a.magic_hw) : m / hw, rem = m - n * hw;
        const int hq = FAST ? fast_div(rem, a.magic_w) : rem / a.Wc, wq = rem - hq * a.Wc;
        c.h0 = a.ph + hq * a.stride + a.pad;
        c.w0 = a.pw + wq * a.stride + a.pad;
        c.base = (int64_t)n * a.Ho * a.Wo * a.K;
    }
    return c;
}

// Element offset of A[m][.] at kernel tap (r,s), channel ch, for forward /
// dgrad; ok = the tap falls inside the image (and, for dgrad, on the stride grid).
template <int MODE>
__device__ __forceinline__ int64_t a_offset_tap(const ConvArgs& a, const RowCtx& c, int r, int s, int ch, bool& ok) {
    if (MODE == CONV_FWD) {
        const int h = c.h0 + r, w = c.w0 + s;
        ok = c.valid && (unsigned)h < (unsigned)a.H && (unsigned)w < (unsigned)a.W;
        return c.base + ((int64_t)r * a.W + s) * a.C + ch;
    } else {
        const int hn = c.h0 - r, wn = c.w0 - s;
        int ho = hn, wo = wn;
        bool on_grid = true;
        if (a.stride == 2) {
            ho = hn >> 1;
            wo = wn >> 1;
            on_grid = ((hn | wn) & 1) == 0;
        } else if (a.stride != 1) {
            ho = hn / a.stride;
            wo = wn / a.stride;
            on_grid = (ho * a.stride == hn) && (wo * a.stride == wn);
        }
        ok = c.valid && hn >= 0 && wn >= 0 && on_grid && ho < a.Ho && wo < a.Wo;
        return c.base + ((int64_t)ho * a.Wo + wo) * a.K + ch;
    }
}

// the same from a flat reduction index (used by the element-wise path only)
template <int MODE>
__device__ __forceinline__ int64_t a_offset(const ConvArgs& a, const RowCtx& c, int kk, bool& ok) {
    const int inner = MODE == CONV_FWD ? a.C : a.K;
    const int tap = kk / inner, ch = kk - tap * inner;
    int r, s;
    if (MODE == CONV_FWD) { r = tap / a.S; s = tap - r * a.S; }
    else { const int ri = tap / a.ns; r = a.r0 + ri * a.stride; s = a.s0 + (tap - ri * a.ns) * a.stride; }
    const int64_t off = a_offset_tap<MODE>(a, c, r, s, ch, ok);
    ok = ok && kk < a.Kred;
    return off;
}

// Vector-path byte offset for forward / dgrad in 32-bit arithmetic (operands
// are below 2 GiB there); tap_off is (r*W + s)*C + ch for the forward pass.
template <int MODE, typename T>
__device__ __forceinline__ unsigned a_voffset(const ConvArgs& a, const RowCtx& c, int r, int s, int ch, int tap_off, bool in_k) {
    if (MODE == CONV_FWD) {
        const int h = c.h0 + r, w = c.w0 + s;
        const bool ok = in_k & c.valid & ((unsigned)h < (unsigned)a.H) & ((unsigned)w < (unsigned)a.W);
        // the offset is formed unconditionally and pushed out of range by its top bit: a select between
        // the two would be compiled into a predicated region, which splits the loop's basic block
        return ((unsigned)((int)c.base + tap_off) * (unsigned)sizeof(T)) | (ok ? 0u : kOutOfRange);
    } else {
        // no branch on the stride (the loop this runs in must stay one basic block): the vector path is taken
        // for strides that are powers of two only.  Negative coordinates are discarded by `ok`.
        const int hn = c.h0 - r, wn = c.w0 - s;
        const int ho = hn >> a.stride_shift, wo = wn >> a.stride_shift;
        const bool on_grid = ((hn | wn) & (a.stride - 1)) == 0;
        const bool ok = in_k & c.valid & ((hn | wn) >= 0) & on_grid & (ho < a.Ho) & (wo < a.Wo);
        return ((unsigned)((int)c.base + (ho * a.Wo + wo) * a.K + ch) * (unsigned)sizeof(T)) | (ok ? 0u : kOutOfRange);
    }
}

// Row of the output matrix a tile row is stored to: the tile row itself, except
// for a residue class of a strided dgrad, whose rows are every stride-th pixel.
template <int MODE, bool FAST = false>
__device__ __forceinline__ int64_t out_row(const ConvArgs& a, int row) {
    if (MODE != CONV_DGRAD || a.stride == 1) return row;
    const int hw = a.Hc * a.Wc;
    const int n = FAST ? fast_div(row, a.magic_hw) : row / hw, rem = row - n * hw;
    const int hq = FAST ? fast_div(rem, a.magic_w) : rem / a.Wc, wq = rem - hq * a.Wc;
    return ((int64_t)n * a.H + a.ph + hq * a.stride) * a.W + a.pw + wq * a.stride;
}

// Tile storage in LDS
//   forward / dgrad: rows of BK reduction elements, padded by one 16-byte vector; a fragment is one
//                    16-byte read (row = lane%32, slice = lane/32).
//   wgrad:           32-bit words [reduction word][row], a word holding the reduction elements 2q, 2q+1
//                    of one row for bf16 (one element for float32); a fragment is four one-word reads,
//                    and the global vectors (channels innermost) go in without any 16-bit scatter.
// FAST: both operands take the 16-byte vector loads and the output width is a
// multiple of a vector, so the kernel has no element-wise paths at all (a
// run-time choice between the two inside the loop would force a wait after
// every load).
template <typename T, int MODE, int WM, int WN, int TM, int TN, int BK, bool FAST, int PF>
__global__ __launch_bounds__(256, 2) void conv_igemm_kernel(ConvArgs a) {   // at least two waves per SIMD: 256 registers
    constexpr bool WG = MODE == CONV_WGRAD;
    constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
    constexpr int VEC = Elem<T>::VEC;
    constexpr int KV = BK / VEC;                    // fwd/dgrad: vectors per tile row
    constexpr int KPD = sizeof(T) == 2 ? 2 : 1;     // wgrad: reduction elements per 32-bit word
    constexpr int KD = BK / KPD;                    // wgrad: words along the reduction
    constexpr int LDPA = BM + 8, LDPB = BN + 8;     // wgrad: words per reduction word-row
    constexpr int RVA = BM / VEC, RVB = BN / VEC;   // wgrad: channel vectors per pixel
    constexpr int TOT_A = WG ? KD * RVA : BM * KV;  // work items per tile (wgrad: KPD vectors each)
    constexpr int TOT_B = WG ? KD * RVB : BN * KV;
    constexpr int ITER_A = (TOT_A + 255) / 256, ITER_B = (TOT_B + 255) / 256;
    constexpr int NRA = WG ? ITER_A * KPD : ITER_A, NRB = WG ? ITER_B * KPD : ITER_B;
    // wgrad in bf16 keeps its tiles as they are in memory, [pixel][channel], and transposes on the way out of
    // LDS (ds_read_tr16_b64, see tr_frag); float32 wgrad keeps words [pixel][channel] read one by one
    constexpr bool WGT = WG && sizeof(T) == 2;
    constexpr bool FRAG_AHEAD = EDL_FRAG_AHEAD != 0 && TM * TN > 1;
    // Tiles loaded straight into LDS: rows of BK elements without padding (RB = 64 or 128 bytes); a wave's load
    // instruction fills 64 consecutive 16-byte slots (whole rows), and the slot of chunk c of row r is
    // c ^ ((r / RPL) % KV) with RPL = rows per 256 bytes, which keeps the fragment reads conflict-free.
    constexpr int RB = BK * (int)sizeof(T), RPL = RB > 256 ? 1 : 256 / RB;
    constexpr bool DIRECT = EDL_DIRECT_LDS != 0 && FAST && !WG && TOT_A % 256 == 0 && TOT_B % 256 == 0 &&
                            (RB == 64 || RB == 128);
    // The bf16 weight gradient the same way: its tiles are rows of pixels as they are in memory, so a
    // wave's load fills whole pixel rows; item v is the 16-byte slot v % RV of pixel v / RV.
    constexpr bool DIRECT_WG = EDL_DIRECT_LDS != 0 && EDL_DIRECT_WG != 0 && FAST && WGT;
    constexpr int DA = DIRECT_WG ? BK * RVA / 256 : 1, DB = DIRECT_WG ? BK * RVB / 256 : 1;   // loads per tile
    static_assert(!DIRECT_WG || (BK * RVA % 256 == 0 && BK * RVB % 256 == 0), "whole waves of slots");
    constexpr bool DMA = DIRECT || DIRECT_WG;
    constexpr int NST = DMA ? PF + 1 : 2;            // LDS stages
    constexpr int LDK = DIRECT ? BK : BK + VEC;
    constexpr int A_STAGE = WGT ? BK * BM * 2 : WG ? KD * LDPA * 4 : BM * LDK * (int)sizeof(T);   // bytes per LDS stage
    constexpr int B_STAGE = WGT ? BK * BN * 2 : WG ? KD * LDPB * 4 : BN * LDK * (int)sizeof(T);
    // epilogue staging: the rows of one wave row, as float32
    constexpr int STAGE_ROWS = TM * 32, STAGE_LD = BN + 4;
    constexpr int TILE_BYTES = NST * (A_STAGE + B_STAGE);
    constexpr int STAGE_BYTES = STAGE_ROWS * STAGE_LD * 4;
    constexpr int SMEM_BYTES = TILE_BYTES > STAGE_BYTES ? TILE_BYTES : STAGE_BYTES;
    static_assert(WM * WN == 4, "four waves per workgroup");
    static_assert(256 % KV == 0 && 256 % RVA == 0 && 256 % RVB == 0, "per-thread column of the tile must be fixed");
    static_assert(!WG || KD == 32, "wgrad: four fragment groups of eight words");

    __shared__ __attribute__((aligned(16))) unsigned char smem[SMEM_BYTES];
    unsigned char* const As = smem;                  // [NST] stages
    unsigned char* const Bs = smem + NST * A_STAGE;

    const T* __restrict__ Ag = (const T*)a.A;
    const T* __restrict__ Bg = (const T*)a.B;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    int tile_x, tile_y, tile_z;
    tile_of_block(a, tile_x, tile_y, tile_z);
    const int m0 = tile_x * BM, n0 = tile_y * BN;
    const int kbeg = tile_z * a.ksplit;
    int kend = kbeg + a.ksplit;
    if (kend > a.Kred) kend = a.Kred;
    const int nk = (kend - kbeg + BK - 1) / BK;

    Vec16<T> ra[PF][NRA], rb[PF][NRB];   // PF register sets: the loads of the next PF tiles are in flight
    const __amdgpu_buffer_rsrc_t rsrcA = make_rsrc(a.A, a.bytesA), rsrcB = make_rsrc(a.B, a.bytesB);
    const i32x4 wordsA = make_rsrc_words(a.A, a.bytesA), wordsB = make_rsrc_words(a.B, a.bytesB);
    // LDS byte address of the 64 slots this wave's first load of a tile fills (DIRECT)
    const unsigned lds_base = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;
    const unsigned ldsA_wave = __builtin_amdgcn_readfirstlane(lds_base + wave * 1024);
    const unsigned ldsB_wave = ldsA_wave + NST * A_STAGE;

    // ---- per-thread state of the gathers; advanced by BK after every tile ------
    RowCtx rowA[WG ? 1 : ITER_A];
    int64_t offB[WG ? 1 : ITER_B];   // fwd/dgrad: start of the weight row
    bool okB[WG ? 1 : ITER_B];
    int tr = 0, ts = 0, tc = 0, tap_off = 0;   // fwd/dgrad: kernel tap and channel of this thread's vector
    int kcur = 0;                    // reduction index of this thread's vector (fwd/dgrad) or of the tile (wgrad)
    constexpr int NOA = DIRECT_WG ? DA : WG ? ITER_A : 1, NPB = DIRECT_WG ? DB : WG ? ITER_B : 1;
    int64_t offA[NOA];               // wgrad: offset of dy[first pixel of the item][first row of the item]
    int pn[NPB], pho[NPB], pwo[NPB]; // wgrad: first pixel of the item
    bool rowA_ok = true;             // wgrad, direct loads: this lane's channels of dy exist
    int wg_r = 0, wg_s = 0, wg_c = 0;  // wgrad: tap and channel of this thread's B rows
    bool wg_j_ok = true;
    int dn = 0, dho = 0, dwo = 0;    // wgrad: BK pixels as (images, rows, columns)
    if (!WG) {
        const int inner = MODE == CONV_FWD ? a.C : a.K;
        // DIRECT: the lane fills slot tid % KV of its rows, which holds chunk slot ^ ((row / RPL) % KV); a lane's
        // rows are 256 / KV apart, so this is the same chunk for all of them
        const int chunk = DIRECT ? ((tid % KV) ^ ((tid / KV / RPL) % KV)) : tid % KV;
        kcur = kbeg + chunk * VEC;
        const int tap = FAST ? fast_div(kcur, a.magic_inner) : kcur / inner;
        tc = kcur - tap * inner;
        if (MODE == CONV_FWD) {
            tr = FAST ? fast_div(tap, a.magic_taps) : tap / a.S;
            ts = tap - tr * a.S;
            tap_off = (tr * a.W + ts) * a.C + tc;
        } else {
            const int ri = FAST ? fast_div(tap, a.magic_taps) : (a.ns > 0 ? tap / a.ns : 0);
            tr = a.r0 + ri * a.stride;
            ts = a.s0 + (tap - ri * a.ns) * a.stride;
            tap_off = (tr * a.S + ts) * a.K + tc;      // position inside a row of the transposed weights
        }
        #pragma unroll
        for (int it = 0; it < ITER_A; ++it) rowA[it] = make_row<MODE, FAST>(a, m0 + (tid + it * 256) / KV);
        #pragma unroll
        for (int it = 0; it < ITER_B; ++it) {
            const int j = n0 + (tid + it * 256) / KV;
            okB[it] = j < a.Nn && (tid + it * 256) < TOT_B;
            offB[it] = (int64_t)j * a.ldb;
        }
    } else if (DIRECT_WG) {
        // slot p of pixel row x holds the 8 channels starting at (((p >> 1) ^ wg_swizzle(x)) << 4) | ((p & 1) << 3)
        // (wg_lds_index); a lane's pixels are a multiple of 4 apart, so its channels are the same in all of them
        const int pa = tid % RVA, pb = tid % RVB;
        const int chA = ((((pa >> 1) ^ wg_swizzle<BM>(tid / RVA)) << 4) | ((pa & 1) << 3));
        const int chB = ((((pb >> 1) ^ wg_swizzle<BN>(tid / RVB)) << 4) | ((pb & 1) << 3));
        rowA_ok = m0 + chA < a.M;
        const int j0 = n0 + chB;
        const int tap = j0 / a.C;
        wg_c = j0 - tap * a.C;
        wg_r = tap / a.S;
        wg_s = tap - wg_r * a.S;
        const int hw = a.Ho * a.Wo;
        dn = BK / hw;
        dho = (BK - dn * hw) / a.Wo;
        dwo = BK - dn * hw - dho * a.Wo;
        #pragma unroll
        for (int it = 0; it < DA; ++it) offA[it] = (int64_t)(kbeg + (tid + it * 256) / RVA) * a.K + m0 + chA;
        #pragma unroll
        for (int it = 0; it < DB; ++it) {
            const int mm = kbeg + (tid + it * 256) / RVB;
            pn[it] = mm / hw;
            const int rem = mm - pn[it] * hw;
            pho[it] = rem / a.Wo;
            pwo[it] = rem - pho[it] * a.Wo;
        }
        wg_j_ok = j0 < a.Nn;
        kcur = kbeg;
    } else {
        const int j0 = n0 + (tid % RVB) * VEC;
        const int tap = j0 / a.C;
        wg_c = j0 - tap * a.C;
        wg_r = tap / a.S;
        wg_s = tap - wg_r * a.S;
        const int hw = a.Ho * a.Wo;
        dn = BK / hw;
        dho = (BK - dn * hw) / a.Wo;
        dwo = BK - dn * hw - dho * a.Wo;
        #pragma unroll
        for (int it = 0; it < ITER_A; ++it)
            offA[it] = (int64_t)(kbeg + ((tid + it * 256) / RVA) * KPD) * a.K + m0 + (tid % RVA) * VEC;
        #pragma unroll
        for (int it = 0; it < ITER_B; ++it) {
            const int mm = kbeg + ((tid + it * 256) / RVB) * KPD;
            pn[it] = mm / hw;
            const int rem = mm - pn[it] * hw;
            pho[it] = rem / a.Wo;
            pwo[it] = rem - pho[it] * a.Wo;
        }
        kcur = kbeg;
    }

    auto load_tiles = [&](int set) {
        if (DIRECT) {
            // `set` is the LDS stage
            const bool in_k = kcur < kend;
            #pragma unroll
            for (int it = 0; it < ITER_A; ++it)
                buffer_load16_to_lds(wordsA, ldsA_wave + set * A_STAGE + it * 4096,
                                     a_voffset<MODE, T>(a, rowA[it], tr, ts, tc, tap_off, in_k));
            #pragma unroll
            for (int it = 0; it < ITER_B; ++it) {
                const int boff = MODE == CONV_FWD ? kcur : tap_off;
                buffer_load16_to_lds(wordsB, ldsB_wave + set * B_STAGE + it * 4096,
                                     (okB[it] && in_k) ? (unsigned)((int)offB[it] + boff) * (unsigned)sizeof(T) : kOutOfRange);
            }
            const int inner = MODE == CONV_FWD ? a.C : a.K;
            kcur += BK;
            const int tap = fast_div(kcur, a.magic_inner);
            tc = kcur - tap * inner;
            const int ri = fast_div(tap, a.magic_taps);
            if (MODE == CONV_FWD) {
                tr = ri;
                ts = tap - ri * a.S;
                tap_off = (tr * a.W + ts) * a.C + tc;
            } else {
                tr = a.r0 + ri * a.stride;
                ts = a.s0 + (tap - ri * a.ns) * a.stride;
                tap_off = (tr * a.S + ts) * a.K + tc;
            }
        } else if (DIRECT_WG) {
            // `set` is the LDS stage; pixel rows past the end of the reduction come in as zeros
            #pragma unroll
            for (int it = 0; it < DA; ++it) {
                const bool ok = rowA_ok & (kcur + (tid + it * 256) / RVA < kend);
                buffer_load16_to_lds(wordsA, ldsA_wave + set * A_STAGE + it * 4096,
                                     ((unsigned)(int)offA[it] * (unsigned)sizeof(T)) | (ok ? 0u : kOutOfRange));
                offA[it] += (int64_t)BK * a.K;
            }
            #pragma unroll
            for (int it = 0; it < DB; ++it) {
                const int h = pho[it] * a.stride - a.pad + wg_r, w = pwo[it] * a.stride - a.pad + wg_s;
                const bool ok = wg_j_ok & (kcur + (tid + it * 256) / RVB < kend) & ((unsigned)h < (unsigned)a.H) &
                                ((unsigned)w < (unsigned)a.W);
                const unsigned off = (unsigned)(((pn[it] * a.H + h) * a.W + w) * a.C + wg_c) * (unsigned)sizeof(T);
                buffer_load16_to_lds(wordsB, ldsB_wave + set * B_STAGE + it * 4096, off | (ok ? 0u : kOutOfRange));
                // advance the item's pixel by BK
                int qw = pwo[it] + dwo, qh = pho[it] + dho, qn = pn[it] + dn;
                const bool cw = qw >= a.Wo;
                qw -= cw ? a.Wo : 0;
                qh += cw ? 1 : 0;
                const bool chh = qh >= a.Ho;
                qh -= chh ? a.Ho : 0;
                qn += chh ? 1 : 0;
                pwo[it] = qw; pho[it] = qh; pn[it] = qn;
            }
            kcur += BK;
        } else if (!WG) {
            const bool in_k = kcur < kend;
            #pragma unroll
            for (int it = 0; it < ITER_A; ++it) {
                ra[set][it].u = make_uint4(0, 0, 0, 0);
                if (TOT_A % 256 != 0 && tid + it * 256 >= TOT_A) continue;
                if (FAST || a.vecA) {
                    ra[set][it].u = buffer_load16(rsrcA, a_voffset<MODE, T>(a, rowA[it], tr, ts, tc, tap_off, in_k));
                } else {
                    #pragma unroll
                    for (int e = 0; e < VEC; ++e) {
                        bool ok;
                        const int64_t off = a_offset<MODE>(a, rowA[it], kcur + e, ok);
                        if (ok && kcur + e < kend) ra[set][it].e[e] = Ag[off];
                    }
                }
            }
            #pragma unroll
            for (int it = 0; it < ITER_B; ++it) {
                rb[set][it].u = make_uint4(0, 0, 0, 0);
                if (FAST || a.vecB) {
                    const int boff = MODE == CONV_FWD ? kcur : tap_off;
                    rb[set][it].u = buffer_load16(rsrcB, (okB[it] && in_k) ? (unsigned)((int)offB[it] + boff) * (unsigned)sizeof(T) : kOutOfRange);
                } else if (okB[it]) {
                    #pragma unroll
                    for (int e = 0; e < VEC; ++e) {
                        int boff = kcur + e;
                        if (MODE == CONV_DGRAD) {
                            const int tap = (kcur + e) / a.K, ri = a.ns > 0 ? tap / a.ns : 0;
                            boff = ((a.r0 + ri * a.stride) * a.S + a.s0 + (tap - ri * a.ns) * a.stride) * a.K + (kcur + e - tap * a.K);
                        }
                        if (kcur + e < kend) rb[set][it].e[e] = Bg[offB[it] + boff];
                    }
                }
            }
            // advance this thread's vector by BK along (r, s, channel); no branches, so that the
            // loads issued above stay in flight across the following code
            const int inner = MODE == CONV_FWD ? a.C : a.K;
            kcur += BK;
            const int tap = fast_div(kcur, a.magic_inner);
            tc = kcur - tap * inner;
            const int ri = fast_div(tap, a.magic_taps);
            if (MODE == CONV_FWD) {
                tr = ri;
                ts = tap - ri * a.S;
                tap_off = (tr * a.W + ts) * a.C + tc;
            } else {
                tr = a.r0 + ri * a.stride;
                ts = a.s0 + (tap - ri * a.ns) * a.stride;
                tap_off = (tr * a.S + ts) * a.K + tc;
            }
        } else {
            #pragma unroll
            for (int it = 0; it < ITER_A; ++it) {
                const bool live = !(TOT_A % 256 != 0 && tid + it * 256 >= TOT_A);
                const int mm = kcur + ((tid + it * 256) / RVA) * KPD;
                const int row0 = m0 + (tid % RVA) * VEC;
                #pragma unroll
                for (int pp = 0; pp < KPD; ++pp) {
                    Vec16<T>& dst = ra[set][it * KPD + pp];
                    dst.u = make_uint4(0, 0, 0, 0);
                    const bool ok = live && mm + pp < kend;
                    if (FAST || a.vecA) {
                        dst.u = buffer_load16(rsrcA, (ok && row0 < a.M) ? (unsigned)((int)offA[it] + pp * a.K) * (unsigned)sizeof(T) : kOutOfRange);
                    } else if (ok) {
                        #pragma unroll
                        for (int e = 0; e < VEC; ++e)
                            if (row0 + e < a.M) dst.e[e] = Ag[offA[it] + (int64_t)pp * a.K + e];
                    }
                }
                offA[it] += (int64_t)BK * a.K;
            }
            #pragma unroll
            for (int it = 0; it < ITER_B; ++it) {
                const bool live = !(TOT_B % 256 != 0 && tid + it * 256 >= TOT_B);
                const int mm = kcur + ((tid + it * 256) / RVB) * KPD;
                int qn = pn[it], qho = pho[it], qwo = pwo[it];
                #pragma unroll
                for (int pp = 0; pp < KPD; ++pp) {
                    Vec16<T>& dst = rb[set][it * KPD + pp];
                    dst.u = make_uint4(0, 0, 0, 0);
                    const bool okp = live && mm + pp < kend;
                    const int hb = qho * a.stride - a.pad, wb = qwo * a.stride - a.pad;
                    if (FAST || a.vecB) {
                        const int j0 = n0 + (tid % RVB) * VEC;
                        const int h = hb + wg_r, w = wb + wg_s;
                        const bool ok = okp && j0 < a.Nn && (unsigned)h < (unsigned)a.H && (unsigned)w < (unsigned)a.W;
                        const unsigned off = (unsigned)(((qn * a.H + h) * a.W + w) * a.C + wg_c) * (unsigned)sizeof(T);
                        dst.u = buffer_load16(rsrcB, ok ? off : kOutOfRange);
                    } else if (okp) {
                        #pragma unroll
                        for (int e = 0; e < VEC; ++e) {
                            const int j = n0 + (tid % RVB) * VEC + e;
                            const int tap = j / a.C, ch = j - tap * a.C;
                            const int r = tap / a.S, s = tap - r * a.S;
                            const int h = hb + r, w = wb + s;
                            if (j < a.Nn && (unsigned)h < (unsigned)a.H && (unsigned)w < (unsigned)a.W)
                                dst.e[e] = Bg[(((int64_t)qn * a.H + h) * a.W + w) * a.C + ch];
                        }
                    }
                    // the next pixel of the pair
                    if (++qwo == a.Wo) { qwo = 0; if (++qho == a.Ho) { qho = 0; ++qn; } }
                }
                // advance the item's first pixel by BK
                pwo[it] += dwo;
                if (pwo[it] >= a.Wo) { pwo[it] -= a.Wo; ++pho[it]; }
                pho[it] += dho;
                if (pho[it] >= a.Ho) { pho[it] -= a.Ho; ++pn[it]; }
                pn[it] += dn;
            }
            kcur += BK;
        }
    };

    auto store_tiles = [&](int set, int buf) {
        if (!WG) {
            T* const Ad = reinterpret_cast<T*>(As + buf * A_STAGE);
            T* const Bd = reinterpret_cast<T*>(Bs + buf * B_STAGE);
            #pragma unroll
            for (int it = 0; it < ITER_A; ++it) {
                const int v = tid + it * 256;
                if (TOT_A % 256 != 0 && v >= TOT_A) continue;
                store_vec(&Ad[(v / KV) * LDK + (v % KV) * VEC], ra[set][it]);
            }
            #pragma unroll
            for (int it = 0; it < ITER_B; ++it) {
                const int v = tid + it * 256;
                if (TOT_B % 256 != 0 && v >= TOT_B) continue;
                store_vec(&Bd[(v / KV) * LDK + (v % KV) * VEC], rb[set][it]);
            }
        } else if (WGT) {
            bf16_t* const Ad = reinterpret_cast<bf16_t*>(As + buf * A_STAGE);
            bf16_t* const Bd = reinterpret_cast<bf16_t*>(Bs + buf * B_STAGE);
            #pragma unroll
            for (int it = 0; it < ITER_A; ++it) {
                const int v = tid + it * 256;
                if (TOT_A % 256 != 0 && v >= TOT_A) continue;
                #pragma unroll
                for (int pp = 0; pp < KPD; ++pp)
                    *reinterpret_cast<uint4*>(&Ad[wg_lds_index<BM>((v / RVA) * KPD + pp, (v % RVA) * VEC)]) = ra[set][it * KPD + pp].u;
            }
            #pragma unroll
            for (int it = 0; it < ITER_B; ++it) {
                const int v = tid + it * 256;
                if (TOT_B % 256 != 0 && v >= TOT_B) continue;
                #pragma unroll
                for (int pp = 0; pp < KPD; ++pp)
                    *reinterpret_cast<uint4*>(&Bd[wg_lds_index<BN>((v / RVB) * KPD + pp, (v % RVB) * VEC)]) = rb[set][it * KPD + pp].u;
            }
        } else {
            uint32_t* const Ad = reinterpret_cast<uint32_t*>(As + buf * A_STAGE);
            uint32_t* const Bd = reinterpret_cast<uint32_t*>(Bs + buf * B_STAGE);
            #pragma unroll
            for (int it = 0; it < ITER_A; ++it) {
                const int v = tid + it * 256;
                if (TOT_A % 256 != 0 && v >= TOT_A) continue;
                uint32_t* dst = &Ad[(v / RVA) * LDPA + (v % RVA) * VEC];
                if (KPD == 2) {
                    // word e = (pixel 2q, pixel 2q+1) of channel e
                    const uint16_t* p0 = reinterpret_cast<const uint16_t*>(&ra[set][it * KPD]);
                    const uint16_t* p1 = reinterpret_cast<const uint16_t*>(&ra[set][it * KPD + KPD - 1]);
                    uint4 lo, hi;
                    lo.x = p0[0] | ((uint32_t)p1[0] << 16); lo.y = p0[1] | ((uint32_t)p1[1] << 16);
                    lo.z = p0[2] | ((uint32_t)p1[2] << 16); lo.w = p0[3] | ((uint32_t)p1[3] << 16);
                    hi.x = p0[4] | ((uint32_t)p1[4] << 16); hi.y = p0[5] | ((uint32_t)p1[5] << 16);
                    hi.z = p0[6] | ((uint32_t)p1[6] << 16); hi.w = p0[7] | ((uint32_t)p1[7] << 16);
                    *reinterpret_cast<uint4*>(dst) = lo;
                    *reinterpret_cast<uint4*>(dst + 4) = hi;
                } else {
                    *reinterpret_cast<uint4*>(dst) = ra[set][it].u;
                }
            }
            #pragma unroll
            for (int it = 0; it < ITER_B; ++it) {
                const int v = tid + it * 256;
                if (TOT_B % 256 != 0 && v >= TOT_B) continue;
                uint32_t* dst = &Bd[(v / RVB) * LDPB + (v % RVB) * VEC];
                if (KPD == 2) {
                    const uint16_t* p0 = reinterpret_cast<const uint16_t*>(&rb[set][it * KPD]);
                    const uint16_t* p1 = reinterpret_cast<const uint16_t*>(&rb[set][it * KPD + KPD - 1]);
                    uint4 lo, hi;
                    lo.x = p0[0] | ((uint32_t)p1[0] << 16); lo.y = p0[1] | ((uint32_t)p1[1] << 16);
                    lo.z = p0[2] | ((uint32_t)p1[2] << 16); lo.w = p0[3] | ((uint32_t)p1[3] << 16);
                    hi.x = p0[4] | ((uint32_t)p1[4] << 16); hi.y = p0[5] | ((uint32_t)p1[5] << 16);
                    hi.z = p0[6] | ((uint32_t)p1[6] << 16); hi.w = p0[7] | ((uint32_t)p1[7] << 16);
                    *reinterpret_cast<uint4*>(dst) = lo;
                    *reinterpret_cast<uint4*>(dst + 4) = hi;
                } else {
                    *reinterpret_cast<uint4*>(dst) = rb[set][it].u;
                }
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

    // Software pipeline: two LDS stages and PF register sets.  While tile k is
    // contracted from LDS stage k%2, the global loads of tiles k+1 .. k+PF are in
    // flight; tile k+1 is moved from its registers to the other stage after the
    // MFMAs of tile k.  One barrier per tile.
    static_assert(DMA || PF == 1 || PF % 2 == 0, "the LDS stage of a tile must be known at compile time");
    // Loads past the end of the reduction are issued too: their offsets are out of
    // range, so they touch no memory and return zeros, and the number of loads in
    // flight at every wait is then a compile-time constant.
    // contraction of the tile in LDS stage `buf`
    auto contract = [&](int buf) {
        constexpr int NG = WG ? 4 : BK / (2 * VEC);   // fragment groups per tile
        auto read_frags = [&](int g, uint4 (&fa)[TM], uint4 (&fb)[TN]) {
            if (!WG) {
                const T* const Ab = reinterpret_cast<const T*>(As + buf * A_STAGE);
                const T* const Bb = reinterpret_cast<const T*>(Bs + buf * B_STAGE);
                // chunk of the row this lane reads, and the slot the tile keeps it in
                const int chunk = 2 * g + (lane >> 5);
                const int slot = DIRECT ? (chunk ^ (((lane & 31) / RPL) % KV)) : chunk;
                #pragma unroll
                for (int i = 0; i < TM; ++i)
                    fa[i] = *reinterpret_cast<const uint4*>(&Ab[((wm * TM + i) * 32 + (lane & 31)) * LDK + slot * VEC]);
                #pragma unroll
                for (int j = 0; j < TN; ++j)
                    fb[j] = *reinterpret_cast<const uint4*>(&Bb[((wn * TN + j) * 32 + (lane & 31)) * LDK + slot * VEC]);
            } else if (WGT) {
                const bf16_t* const Ab = reinterpret_cast<const bf16_t*>(As + buf * A_STAGE);
                const bf16_t* const Bb = reinterpret_cast<const bf16_t*>(Bs + buf * B_STAGE);
                #pragma unroll
                for (int i = 0; i < TM; ++i) fa[i] = tr_frag<BM>(Ab, (wm * TM + i) * 32, g * 16, lane);
                #pragma unroll
                for (int j = 0; j < TN; ++j) fb[j] = tr_frag<BN>(Bb, (wn * TN + j) * 32, g * 16, lane);
            } else {
                const uint32_t* const Ab = reinterpret_cast<const uint32_t*>(As + buf * A_STAGE) + (g * 8 + (lane >> 5) * 4) * LDPA + (lane & 31);
                const uint32_t* const Bb = reinterpret_cast<const uint32_t*>(Bs + buf * B_STAGE) + (g * 8 + (lane >> 5) * 4) * LDPB + (lane & 31);
                #pragma unroll
                for (int i = 0; i < TM; ++i) {
                    const uint32_t* q = Ab + (wm * TM + i) * 32;
                    fa[i] = make_uint4(q[0], q[LDPA], q[2 * LDPA], q[3 * LDPA]);
                }
                #pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const uint32_t* q = Bb + (wn * TN + j) * 32;
                    fb[j] = make_uint4(q[0], q[LDPB], q[2 * LDPB], q[3 * LDPB]);
                }
            }
        };
        // The fragments of group g+1 are read from LDS before the MFMAs of group g are issued
        // (the fences keep the compiler from sinking the reads back to their first use), so the
        // LDS latency of one group hides behind the matrix work of the one before.
        uint4 fa[2][TM], fb[2][TN];
        read_frags(0, fa[0], fb[0]);
        #pragma unroll
        for (int g = 0; g < NG; ++g) {
            if (g + 1 < NG) read_frags(g + 1, fa[(g + 1) & 1], fb[(g + 1) & 1]);
            if (FRAG_AHEAD) __builtin_amdgcn_sched_barrier(0);
            #pragma unroll
            for (int i = 0; i < TM; ++i)
                #pragma unroll
                for (int j = 0; j < TN; ++j) Frag<T>::mma(fa[g & 1][i], fb[g & 1][j], acc[i][j]);
            if (FRAG_AHEAD) __builtin_amdgcn_sched_barrier(0);
        }
    };
    if (DMA) {
        // NST LDS stages filled by direct loads, no registers in between: while tile k is contracted from
        // stage k % NST, the loads of tiles k+1 .. k+NST-1 are in flight.  Per tile: wait until this wave's
        // loads of tile k have landed (loads complete in order, so all but those of the NST-2 younger tiles),
        // barrier (every wave's part of tile k is in LDS and every wave is done reading tile k-1), then
        // refill the stage tile k-1 was in.  Loads past the end of the reduction write zeros into a stage
        // nobody reads; all of them have landed before the epilogue reuses the memory.
        constexpr int PER_TILE = DIRECT_WG ? DA + DB : ITER_A + ITER_B;
        #pragma unroll
        for (int u = 0; u < NST - 1; ++u) load_tiles(u);
        for (int kt = 0; kt < nk; kt += NST) {
            #pragma unroll
            for (int u = 0; u < NST; ++u) {
                if (kt + u >= nk) break;
                wait_vmcnt<(NST - 2) * PER_TILE>();
                __syncthreads();
                load_tiles((u + NST - 1) % NST);
                contract(u);
            }
        }
        wait_vmcnt<0>();
        __syncthreads();
    } else {
        #pragma unroll
        for (int u = 0; u < PF; ++u) load_tiles(u);
        store_tiles(0, 0);
        __syncthreads();
        for (int kt = 0; kt < nk; kt += PF) {
            #pragma unroll
            for (int u = 0; u < PF; ++u) {
                const int k = kt + u;
                if (k >= nk) break;
                const int buf = PF == 1 ? (k & 1) : (u & 1);
                load_tiles(u);
                contract(buf);
                store_tiles((u + 1) % PF, buf ^ 1);
                __syncthreads();
            }
        }
    }

    // ---- epilogue: lane holds column lane%32, rows (q/4)*8 + (lane/32)*4 + q%4 of each 32x32 tile ----
    constexpr bool OUT_F32 = WG || sizeof(T) == 4;       // element type of the vector-path output
    constexpr int OSZ = OUT_F32 ? 4 : 2;
    constexpr int OVEC = 16 / OSZ;
    if (!FAST) {
        // ragged width (or float32 logits from a bf16 net): element-wise stores
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
                        const int64_t o = out_row<MODE>(a, row) * a.Nn + col;
                        T* dst = (T*)a.out;
                        if (a.accumulate) v += Elem<T>::to_f32(a.acc_src ? ((const T*)a.acc_src)[o] : dst[o]);
                        dst[o] = Elem<T>::from_f32(v);
                    } else {
                        ((float*)a.out)[((int64_t)tile_z * a.M + row) * a.Nn + col] = v;
                    }
                }
            }
        }
        return;
    }
    // staged: one wave row at a time goes through LDS as float32 (one word per
    // lane and row, conflict-free), then leaves as 16-byte vectors along the output row
    float* const stage = reinterpret_cast<float*>(smem);
    unsigned char* const outp = (unsigned char*)a.out + (WG ? (int64_t)tile_z * a.M * a.Nn * 4 : 0);
    const unsigned char* const accp = (MODE == CONV_DGRAD && a.acc_src != nullptr) ? (const unsigned char*)a.acc_src : outp;
    const bool to_partial = !WG && a.partial != nullptr;     // cut reduction: raw float32 sums, finished by another kernel
    const bool f32_out = (MODE == CONV_FWD) && a.out_fp32 && !OUT_F32;
    // Every lane stores the same OVEC columns in each of its rows (256 is a multiple of the
    // vectors per row), so column sums of what it stored stay in registers until the end.
    const bool with_stats = MODE == CONV_FWD && a.stats != nullptr;
    float csum[OVEC], csq[OVEC];
    #pragma unroll
    for (int e = 0; e < OVEC; ++e) csum[e] = csq[e] = 0.f;
    constexpr int CV = BN / OVEC;                              // vectors per stored row
    constexpr int NV = (STAGE_ROWS * CV + 255) / 256;          // vectors per lane and pass
    const bool add_old = MODE == CONV_DGRAD && a.accumulate && !to_partial;
    const bool masked = MODE == CONV_DGRAD && a.mask_act != nullptr && !to_partial;
    const bool with_xhat = masked && a.xin != nullptr;
    float mu[OVEC], rs[OVEC];      // of this lane's columns
    #pragma unroll
    for (int e = 0; e < OVEC; ++e) { mu[e] = 0.f; rs[e] = 0.f; }
    if (with_xhat) {
        const int c0 = n0 + (tid % CV) * OVEC;
        #pragma unroll
        for (int e = 0; e < OVEC; ++e)
            if (c0 + e < a.Nn) { mu[e] = a.mean_rstd[c0 + e]; rs[e] = a.mean_rstd[a.Nn + c0 + e]; }
    }
    #pragma unroll
    for (int pass = 0; pass < WM; ++pass) {
        // dgrad adding to an existing gradient: its vectors are fetched now, all at once and without a
        // branch (a vector outside the matrix reads the start of the tensor and is ignored), and are
        // there when the staged sums are
        uint4 oldv[NV];
        if (add_old) {
            #pragma unroll
            for (int k = 0; k < NV; ++k) {
                const int v = tid + k * 256, rl = v / CV, cv = v - rl * CV;
                const int row = m0 + pass * STAGE_ROWS + rl, col = n0 + cv * OVEC;
                const bool inside = v < STAGE_ROWS * CV && row < a.M && col < a.Nn;
                const unsigned char* src = inside ? accp + (out_row<MODE, true>(a, row) * a.Nn + col) * OSZ : accp;
                oldv[k] = *reinterpret_cast<const uint4*>(src);
            }
        }
        // the activation (and the batch norm's input) at the positions this lane stores, fetched the same way
        uint4 actv[NV], xinv[NV];
        if (masked) {
            #pragma unroll
            for (int k = 0; k < NV; ++k) {
                const int v = tid + k * 256, rl = v / CV, cv = v - rl * CV;
                const int row = m0 + pass * STAGE_ROWS + rl, col = n0 + cv * OVEC;
                const bool inside = v < STAGE_ROWS * CV && row < a.M && col < a.Nn;
                const int64_t at = inside ? ((int64_t)row * a.Nn + col) * OSZ : 0;
                actv[k] = *reinterpret_cast<const uint4*>((const unsigned char*)a.mask_act + at);
                if (with_xhat) xinv[k] = *reinterpret_cast<const uint4*>((const unsigned char*)a.xin + at);
            }
        }
        if (wm == pass) {
            #pragma unroll
            for (int i = 0; i < TM; ++i) {
                #pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const int cl = (wn * TN + j) * 32 + (lane & 31);
                    const int col = n0 + cl;
                    const float bias = (MODE == CONV_FWD && a.bias && col < a.Nn) ? a.bias[col] : 0.f;
                    float* sp = stage + (i * 32 + (lane >> 5) * 4) * STAGE_LD + cl;
                    #pragma unroll
                    for (int q = 0; q < 16; ++q) {
                        float v = acc[i][j][q];
                        if (MODE == CONV_FWD && !to_partial) {
                            v += bias;
                            if (a.relu) v = fmaxf(v, 0.f);
                        }
                        sp[((q >> 2) * 8 + (q & 3)) * STAGE_LD] = v;
                    }
                }
            }
        }
        __syncthreads();
        #pragma unroll
        for (int k = 0; k < NV; ++k) {
            const int v = tid + k * 256;
            if (v >= STAGE_ROWS * CV) break;
            const int rl = v / CV, cv = v - rl * CV;
            const int row = m0 + pass * STAGE_ROWS + rl, col = n0 + cv * OVEC;
            if (row < a.M && col < a.Nn) {
                const float* sp = stage + rl * STAGE_LD + cv * OVEC;
                if (to_partial || f32_out) {
                    float* d = to_partial ? a.partial + ((int64_t)tile_z * a.M + row) * a.Nn + col
                                          : (float*)a.out + (int64_t)row * a.Nn + col;
                    #pragma unroll
                    for (int e = 0; e < OVEC; e += 4) *reinterpret_cast<float4*>(d + e) = *reinterpret_cast<const float4*>(sp + e);
                    continue;
                }
                unsigned char* dst = outp + (out_row<MODE, true>(a, row) * a.Nn + col) * OSZ;
                if (OUT_F32) {
                    float4 o = *reinterpret_cast<const float4*>(sp);
                    if (add_old) {
                        o.x += __uint_as_float(oldv[k].x); o.y += __uint_as_float(oldv[k].y);
                        o.z += __uint_as_float(oldv[k].z); o.w += __uint_as_float(oldv[k].w);
                    }
                    if (masked) {
                        const float am[4] = {__uint_as_float(actv[k].x), __uint_as_float(actv[k].y), __uint_as_float(actv[k].z), __uint_as_float(actv[k].w)};
                        o.x = am[0] > 0.f ? o.x : 0.f; o.y = am[1] > 0.f ? o.y : 0.f;
                        o.z = am[2] > 0.f ? o.z : 0.f; o.w = am[3] > 0.f ? o.w : 0.f;
                        const float gv[4] = {o.x, o.y, o.z, o.w};
                        const float xv[4] = {__uint_as_float(xinv[k].x), __uint_as_float(xinv[k].y), __uint_as_float(xinv[k].z), __uint_as_float(xinv[k].w)};
                        #pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            csum[e % OVEC] += gv[e];
                            if (with_xhat) csq[e % OVEC] += gv[e] * ((xv[e] - mu[e % OVEC]) * rs[e % OVEC]);
                        }
                    }
                    *reinterpret_cast<float4*>(dst) = o;
                    if (with_stats) {
                        csum[0] += o.x; csq[0] += o.x * o.x; csum[1] += o.y; csq[1] += o.y * o.y;
                        csum[2] += o.z; csq[2] += o.z * o.z; csum[3] += o.w; csq[3] += o.w * o.w;
                    }
                } else {
                    float4 o0 = *reinterpret_cast<const float4*>(sp), o1 = *reinterpret_cast<const float4*>(sp + 4);
                    if (add_old) {
                        const uint4 old = oldv[k];
                        o0.x += __uint_as_float(old.x << 16); o0.y += __uint_as_float(old.x & 0xffff0000u);
                        o0.z += __uint_as_float(old.y << 16); o0.w += __uint_as_float(old.y & 0xffff0000u);
                        o1.x += __uint_as_float(old.z << 16); o1.y += __uint_as_float(old.z & 0xffff0000u);
                        o1.z += __uint_as_float(old.w << 16); o1.w += __uint_as_float(old.w & 0xffff0000u);
                    }
                    if (masked) {   // activation > 0: a positive bf16 (sign clear, not zero)
                        const uint32_t aw[4] = {actv[k].x, actv[k].y, actv[k].z, actv[k].w};
                        float* const ov[8] = {&o0.x, &o0.y, &o0.z, &o0.w, &o1.x, &o1.y, &o1.z, &o1.w};
                        #pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            if (!(__uint_as_float(aw[e] << 16) > 0.f)) *ov[2 * e] = 0.f;
                            if (!(__uint_as_float(aw[e] & 0xffff0000u) > 0.f)) *ov[2 * e + 1] = 0.f;
                        }
                    }
                    uint4 pk;
                    pk.x = pack2_bf16(o0.x, o0.y); pk.y = pack2_bf16(o0.z, o0.w);
                    pk.z = pack2_bf16(o1.x, o1.y); pk.w = pack2_bf16(o1.z, o1.w);
                    *reinterpret_cast<uint4*>(dst) = pk;
                    if (masked) {   // sums of the stored (rounded) gradient
                        const uint32_t w4[4] = {pk.x, pk.y, pk.z, pk.w};
                        const uint32_t xw[4] = {xinv[k].x, xinv[k].y, xinv[k].z, xinv[k].w};
                        #pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float lo = __uint_as_float(w4[e] << 16), hi = __uint_as_float(w4[e] & 0xffff0000u);
                            csum[(2 * e) % OVEC] += lo;
                            csum[(2 * e + 1) % OVEC] += hi;
                            if (with_xhat) {
                                const float xl = __uint_as_float(xw[e] << 16), xh = __uint_as_float(xw[e] & 0xffff0000u);
                                csq[(2 * e) % OVEC] += lo * ((xl - mu[(2 * e) % OVEC]) * rs[(2 * e) % OVEC]);
                                csq[(2 * e + 1) % OVEC] += hi * ((xh - mu[(2 * e + 1) % OVEC]) * rs[(2 * e + 1) % OVEC]);
                            }
                        }
                    }
                    if (with_stats) {   // of the rounded values, as a reader of the stored tensor would see them
                        const uint32_t w4[4] = {pk.x, pk.y, pk.z, pk.w};
                        #pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float lo = __uint_as_float(w4[e] << 16), hi = __uint_as_float(w4[e] & 0xffff0000u);
                            csum[(2 * e) % OVEC] += lo; csq[(2 * e) % OVEC] += lo * lo;
                            csum[(2 * e + 1) % OVEC] += hi; csq[(2 * e + 1) % OVEC] += hi * hi;
                        }
                    }
                }
            }
        }
        __syncthreads();
    }
    if (with_stats || masked) {
        float* const sums = with_stats ? a.stats : a.msum;
        // lanes with the same column vector differ in tid / CV: sum over them in a fixed order
        constexpr int GROUPS = 256 / CV;
        static_assert(2 * GROUPS * BN * 4 <= SMEM_BYTES, "column sums fit the tile memory");
        float* const red = stage;
        const int grp = tid / CV, c0 = (tid % CV) * OVEC;
        #pragma unroll
        for (int e = 0; e < OVEC; ++e) {
            red[grp * BN + c0 + e] = csum[e];
            red[(GROUPS + grp) * BN + c0 + e] = csq[e];
        }
        __syncthreads();
        for (int c = tid; c < BN; c += 256) {
            if (n0 + c >= a.Nn) continue;
            float s1 = 0.f, s2 = 0.f;
            #pragma unroll 8
            for (int gq = 0; gq < GROUPS; ++gq) { s1 += red[gq * BN + c]; s2 += red[(GROUPS + gq) * BN + c]; }
            sums[(int64_t)(n0 + c) * a.red_stride + tile_x] = s1;
            sums[(int64_t)(a.Nn + n0 + c) * a.red_stride + tile_x] = s2;
        }
    }
}

// dw[i] = sum over splits, in split order.  One 16-byte vector per lane and
// split (the splits' loads are independent, so they are all in flight together).
template <int VECW>
__global__ __launch_bounds__(256) void wgrad_reduce_kernel(const float* __restrict__ part, float* __restrict__ dw, int64_t n,
                                                           int splits) {
    const int64_t nv = n / VECW;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < nv; i += stride) {
        if (VECW == 4) {
            float4 s = reinterpret_cast<const float4*>(part)[i];
            int k = 1;
            for (; k + 3 < splits; k += 4) {
                const float4 t0 = reinterpret_cast<const float4*>(part + (int64_t)k * n)[i];
                const float4 t1 = reinterpret_cast<const float4*>(part + (int64_t)(k + 1) * n)[i];
                const float4 t2 = reinterpret_cast<const float4*>(part + (int64_t)(k + 2) * n)[i];
                const float4 t3 = reinterpret_cast<const float4*>(part + (int64_t)(k + 3) * n)[i];
                s.x += t0.x; s.y += t0.y; s.z += t0.z; s.w += t0.w;
                s.x += t1.x; s.y += t1.y; s.z += t1.z; s.w += t1.w;
                s.x += t2.x; s.y += t2.y; s.z += t2.z; s.w += t2.w;
                s.x += t3.x; s.y += t3.y; s.z += t3.z; s.w += t3.w;
            }
            for (; k < splits; ++k) {
                const float4 t = reinterpret_cast<const float4*>(part + (int64_t)k * n)[i];
                s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
            }
            reinterpret_cast<float4*>(dw)[i] = s;
        } else {
            float s = part[i];
            for (int k = 1; k < splits; ++k) s += part[(int64_t)k * n + i];
            dw[i] = s;
        }
    }
}

// Finish of a forward / dgrad whose reduction was cut: sum the splits in order,
// add the bias / apply ReLU (forward) or add the existing gradient (dgrad), and
// store in the output type.  Four outputs per lane.
template <typename T, bool MASKED>
__global__ __launch_bounds__(256) void splitk_finish_kernel(const float* __restrict__ part, void* out, const float* __restrict__ bias,
                                                            int64_t M, int Nn, int splits, int relu, int out_fp32, int accumulate,
                                                            int rows_per_block, float* __restrict__ stats,
                                                            const T* __restrict__ mask_act, const T* __restrict__ xin,
                                                            const float* __restrict__ mean_rstd, const void* acc_src) {
    if (acc_src == nullptr) acc_src = out;      // where the gradient that is added to is read (see ConvArgs)
    // a workgroup owns 64 columns of rows_per_block rows: 16 lanes across (4 columns each), 16 rows at a time
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int col = (blockIdx.x * 16 + tx) * 4;
    const bool active = col < Nn;
    const int64_t mn = M * Nn;
    const int64_t r0 = (int64_t)blockIdx.y * rows_per_block;
    int64_t r1 = r0 + rows_per_block;
    if (r1 > M) r1 = M;
    float4 bv = make_float4(0.f, 0.f, 0.f, 0.f);
    if (bias && active) bv = *reinterpret_cast<const float4*>(bias + col);
    float cs[4] = {0.f, 0.f, 0.f, 0.f}, cq[4] = {0.f, 0.f, 0.f, 0.f};
    // MASKED (input gradient): the sum is stored where the activation is positive, zero elsewhere, and the
    // column sums are those of the stored gradient and of gradient x normalised input (with xin)
    float mu[4] = {0.f, 0.f, 0.f, 0.f}, rs[4] = {0.f, 0.f, 0.f, 0.f};
    if (MASKED && xin != nullptr && active) {
        #pragma unroll
        for (int e = 0; e < 4; ++e) { mu[e] = mean_rstd[col + e]; rs[e] = mean_rstd[Nn + col + e]; }
    }
    if (active) {
        for (int64_t r = r0 + ty; r < r1; r += 16) {
            const int64_t i = r * Nn + col;
            float4 s = *reinterpret_cast<const float4*>(part + i);
            for (int k = 1; k < splits; ++k) {
                const float4 t = *reinterpret_cast<const float4*>(part + (int64_t)k * mn + i);
                s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
            }
            s.x += bv.x; s.y += bv.y; s.z += bv.z; s.w += bv.w;
            if (relu) { s.x = fmaxf(s.x, 0.f); s.y = fmaxf(s.y, 0.f); s.z = fmaxf(s.z, 0.f); s.w = fmaxf(s.w, 0.f); }
            if (out_fp32 || sizeof(T) == 4) {
                float4* d = reinterpret_cast<float4*>((float*)out + i);
                if (accumulate) {
                    const float4 o = *reinterpret_cast<const float4*>((const float*)acc_src + i);
                    s.x += o.x; s.y += o.y; s.z += o.z; s.w += o.w;
                }
                if (MASKED) {
                    const float4 am = *reinterpret_cast<const float4*>((const float*)mask_act + i);
                    s.x = am.x > 0.f ? s.x : 0.f; s.y = am.y > 0.f ? s.y : 0.f;
                    s.z = am.z > 0.f ? s.z : 0.f; s.w = am.w > 0.f ? s.w : 0.f;
                }
                *d = s;
                if (MASKED) {
                    float4 xv = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (xin != nullptr) xv = *reinterpret_cast<const float4*>((const float*)xin + i);
                    cs[0] += s.x; cs[1] += s.y; cs[2] += s.z; cs[3] += s.w;
                    if (xin != nullptr) {
                        cq[0] += s.x * ((xv.x - mu[0]) * rs[0]); cq[1] += s.y * ((xv.y - mu[1]) * rs[1]);
                        cq[2] += s.z * ((xv.z - mu[2]) * rs[2]); cq[3] += s.w * ((xv.w - mu[3]) * rs[3]);
                    }
                    continue;
                }
            } else {
                uint2* d = reinterpret_cast<uint2*>((bf16_t*)out + i);
                if (accumulate) {
                    const uint2 o = *reinterpret_cast<const uint2*>((const bf16_t*)acc_src + i);
                    s.x += __uint_as_float(o.x << 16); s.y += __uint_as_float(o.x & 0xffff0000u);
                    s.z += __uint_as_float(o.y << 16); s.w += __uint_as_float(o.y & 0xffff0000u);
                }
                if (MASKED) {   // activation > 0: a positive bf16
                    const uint2 am = *reinterpret_cast<const uint2*>((const bf16_t*)mask_act + i);
                    if (!(__uint_as_float(am.x << 16) > 0.f)) s.x = 0.f;
                    if (!(__uint_as_float(am.x & 0xffff0000u) > 0.f)) s.y = 0.f;
                    if (!(__uint_as_float(am.y << 16) > 0.f)) s.z = 0.f;
                    if (!(__uint_as_float(am.y & 0xffff0000u) > 0.f)) s.w = 0.f;
                }
                const uint2 pk = make_uint2(pack2_bf16(s.x, s.y), pack2_bf16(s.z, s.w));
                *d = pk;
                // what a reader of the stored tensor sees
                s.x = __uint_as_float(pk.x << 16); s.y = __uint_as_float(pk.x & 0xffff0000u);
                s.z = __uint_as_float(pk.y << 16); s.w = __uint_as_float(pk.y & 0xffff0000u);
                if (MASKED) {
                    uint2 xw = make_uint2(0u, 0u);
                    if (xin != nullptr) xw = *reinterpret_cast<const uint2*>((const bf16_t*)xin + i);
                    const float x0 = __uint_as_float(xw.x << 16), x1 = __uint_as_float(xw.x & 0xffff0000u);
                    const float x2 = __uint_as_float(xw.y << 16), x3 = __uint_as_float(xw.y & 0xffff0000u);
                    cs[0] += s.x; cs[1] += s.y; cs[2] += s.z; cs[3] += s.w;
                    if (xin != nullptr) {
                        cq[0] += s.x * ((x0 - mu[0]) * rs[0]); cq[1] += s.y * ((x1 - mu[1]) * rs[1]);
                        cq[2] += s.z * ((x2 - mu[2]) * rs[2]); cq[3] += s.w * ((x3 - mu[3]) * rs[3]);
                    }
                    continue;
                }
            }
            cs[0] += s.x; cq[0] += s.x * s.x; cs[1] += s.y; cq[1] += s.y * s.y;
            cs[2] += s.z; cq[2] += s.z * s.z; cs[3] += s.w; cq[3] += s.w * s.w;
        }
    }
    if (stats == nullptr) return;
    // column sums of the stored values and of their squares, per row block (the batch-norm reduction's layout)
    __shared__ float red[2][16][64 + 1];
    #pragma unroll
    for (int e = 0; e < 4; ++e) { red[0][ty][tx * 4 + e] = cs[e]; red[1][ty][tx * 4 + e] = cq[e]; }
    __syncthreads();
    if (threadIdx.x < 128) {
        const int kind = threadIdx.x >> 6, c = threadIdx.x & 63, cg = blockIdx.x * 64 + c;
        if (cg < Nn) {
            float t = 0.f;
            #pragma unroll
            for (int j = 0; j < 16; ++j) t += red[kind][j][c];
            stats[(int64_t)(kind * Nn + cg) * kRedRowBlocks + blockIdx.y] = t;
        }
    }
}

// ---------------------------------------------------------------------------
// host side: tile selection and launch
// ---------------------------------------------------------------------------
enum TileCfg { T128x128, T128x64, T128x32, T64x64 };

#ifndef EDL_PF_BIG
#define EDL_PF_BIG 1
#endif
#ifndef EDL_PF_SMALL
#define EDL_PF_SMALL 2
#endif
#ifndef EDL_BK_SMALL_MULT
#define EDL_BK_SMALL_MULT 1
#endif
#ifndef EDL_BK_BIG_DIV
#define EDL_BK_BIG_DIV 2
#endif
#ifndef EDL_BK_SMALL_DIV
#define EDL_BK_SMALL_DIV 1
#endif
#ifndef EDL_PF_BIG_HALF
#define EDL_PF_BIG_HALF EDL_PF_BIG
#endif
#ifndef EDL_PF_SMALL_TAIL
#define EDL_PF_SMALL_TAIL 1
#endif
#ifndef EDL_PF_WG_BIG
#define EDL_PF_WG_BIG EDL_PF_BIG
#endif
#ifndef EDL_PF_WG_DEEP
#define EDL_PF_WG_DEEP 2
#endif
#ifndef EDL_PF_WG_SMALL
#define EDL_PF_WG_SMALL 2
#endif

// reduction elements per tile: eight 16-byte vectors per row for either type
template <typename T> constexpr int kConvBK = 8 * Elem<T>::VEC;

// short_fwd: a problem whose epilogue is most of the workgroup's time (a forward pass of one or two
// reduction steps, an input-gradient pass whose epilogue adds, masks and sums); twice as many workgroups of
// half the width measured faster there
static TileCfg pick_tile(int M, int Nn, int Kred, int* bm, int* bn, bool short_fwd = false) {
    // A long reduction takes the 128x128 tile from fewer tiles on (the reduction is cut to fill the chip):
    // VGG-16's 14x14 layers, 196 tiles, measured 64 -> 48 us forward and 71 -> 47 us dgrad.
    const int min128_short = (int)tune().min128, min128_long = (int)tune().min128_long;
    const int min128 = Kred >= 4096 ? std::min(min128_short, min128_long) : min128_short;
    TileCfg t;
    if (Nn <= 32) t = T128x32;
    else if (Nn <= 64) t = (M >= 128) ? T128x64 : T64x64;
    else {
        const int64_t tiles = (int64_t)((M + 127) / 128) * ((Nn + 127) / 128);
        t = (tiles >= min128 && M >= 128) ? (short_fwd ? T128x64 : T128x128) : T64x64;
    }
    // measurement aid: one tile shape for every forward / dgrad problem it fits (0..3 = 128x128, 128x64, 128x32, 64x64)
    const int force = (int)tune().force_tile;
    if (force >= 0 && force <= 3) t = (TileCfg)force;
    switch (t) {
        case T128x128: *bm = 128; *bn = 128; break;
        case T128x64: *bm = 128; *bn = 64; break;
        case T128x32: *bm = 128; *bn = 32; break;
        default: *bm = 64; *bn = 64; break;
    }
    return t;
}

static unsigned long long magic_of(int d) {
    if (d <= 0) return 0;
    return ((1ull << 40) + (unsigned long long)d - 1) / (unsigned long long)d;
}

// n / d == (n * magic_of(d)) >> 40 for every 0 <= n <= n_max: the error term needs n * d < 2^40 and the
// product must fit 64 bits
static bool magic_fits(double n_max, int d) {
    if (d <= 0) return true;
    return n_max * (double)d < 1.0e12 && n_max * (double)magic_of(d) < 9.0e18;
}

template <typename T, int MODE>
static void launch_cfg(TileCfg t, bool fast, dim3 tiles, const ConvArgs& a_in, hipStream_t st) {
    constexpr int BK = kConvBK<T>;
    ConvArgs a = a_in;
    a.gx = (int)tiles.x; a.gy = (int)tiles.y; a.gz = (int)tiles.z;
    const double total = (double)a.gx * a.gy * a.gz;
    const bool mg = magic_fits(total, a.gx) && magic_fits(total, a.gy);
    a.magic_gx = mg ? magic_of(a.gx) : 0; a.magic_gy = mg ? magic_of(a.gy) : 0;
    const dim3 grid(tiles.x * tiles.y * tiles.z);
    // Measured on ResNet-50 at a shard of 32: the 64x64 tile (few registers per set, the least MFMA work per
    // reduction step, often fewer workgroups than the chip has room for) gains a third on long reductions from
    // two register sets of loads in flight; the 128-wide tiles gain nothing from a second set but do from
    // half-length reduction steps (half the LDS per workgroup, so more workgroups per CU).
    constexpr int PF_BIG = EDL_PF_BIG, PF_SMALL = MODE == CONV_WGRAD ? EDL_PF_WG_SMALL : EDL_PF_SMALL;
    constexpr int PF_HALF = MODE == CONV_WGRAD ? EDL_PF_WG_BIG : EDL_PF_BIG_HALF;   // 128-wide tiles on half-length steps
    constexpr int BK_SMALL = MODE == CONV_WGRAD ? BK : EDL_BK_SMALL_MULT * BK / EDL_BK_SMALL_DIV;
    constexpr int BK_BIG = MODE == CONV_WGRAD ? BK : BK / EDL_BK_BIG_DIV;
    // A weight gradient of at most one workgroup per CU has nobody to take turns with: one more tile in flight
    // hides the operand latency its single wave per SIMD leaves exposed (bf16; ResNet-50 at a shard of 32: 128x128 tiles
    // 22.2 -> 20.1 us, 128x64 24.4 -> 18.4 us).  Launches of more workgroups than CUs (VGG-16's long reductions, cut
    // into two workgroups per CU) keep the two-stage form: with a third stage only one workgroup fits a CU's LDS
    // (73.7 -> 113 us).
    constexpr int PF_DEEP = MODE == CONV_WGRAD ? EDL_PF_WG_DEEP : PF_BIG;
    const bool deep = MODE == CONV_WGRAD && total <= (double)tune().wgrad_deep_max;
    if (!fast) {   // element-wise kernel: one tile shape only
        hipLaunchKernelGGL((conv_igemm_kernel<T, MODE, 2, 2, 1, 1, BK, false, 1>), grid, dim3(256), 0, st, a);
        return;
    }
    switch (t) {
        case T128x128: {
            // Long reductions (VGG-16's 3x3 layers: 1,152 to 4,608 elements) run faster on full-length reduction
            // steps (half the barriers per MFMA: measured 159 -> 135 us forward, 174 -> 154 us dgrad on VGG-16);
            // short ones (ResNet-50's 1x1 layers) want the smaller LDS footprint and more workgroups per CU.
            const int full_steps_from = (int)tune().bk64_kred;
            if constexpr (MODE == CONV_WGRAD && sizeof(T) == 2) {
                if (deep) {
                    hipLaunchKernelGGL((conv_igemm_kernel<T, MODE, 2, 2, 2, 2, BK, true, PF_DEEP>), grid, dim3(256), 0, st, a);
                    break;
                }
            }
            if (BK_BIG != BK && a.Kred >= full_steps_from)
                hipLaunchKernelGGL((conv_igemm_kernel<T, MODE, 2, 2, 2, 2, BK, true, PF_BIG>), grid, dim3(256), 0, st, a);
            else
                hipLaunchKernelGGL((conv_igemm_kernel<T, MODE, 2, 2, 2, 2, BK_BIG, true, PF_HALF>), grid, dim3(256), 0, st, a);
            break;
        }
        case T128x64:
            if constexpr (MODE == CONV_WGRAD && sizeof(T) == 2) {
                if (deep) {
                    hipLaunchKernelGGL((conv_igemm_kernel<T, MODE, 2, 2, 2, 1, BK, true, PF_DEEP>), grid, dim3(256), 0, st, a);
                    break;
                }
            }
            hipLaunchKernelGGL((conv_igemm_kernel<T, MODE, 2, 2, 2, 1, BK_BIG, true, PF_HALF>), grid, dim3(256), 0, st, a);
            break;
        case T128x32: hipLaunchKernelGGL((conv_igemm_kernel<T, MODE, 4, 1, 1, 1, BK, true, PF_BIG>), grid, dim3(256), 0, st, a); break;
        default:
            if constexpr (MODE != CONV_WGRAD && sizeof(T) == 2) {
                // Three stages of a 64x64 tile are 48 KB of LDS: three workgroups per CU, 768 on the chip.  A launch
                // of a few more (784 and 800 are common: 25,088 pixels x 128 channels, 1,568 x 2,048) ran a second
                // round for its last 16 or 32 workgroups and took almost twice one round.  Such launches run the
                // two-stage form (32 KB, five per CU), so that all of their workgroups are resident at once:
                // 22.1 -> 18.2 us and 25.9 -> 22.2 us for the 3x3 layers at 28x28, 0.490 -> 0.422 ms per ResNet-50
                // step over all launches of that size.
                if (total > (double)tune().small_tail_from && total <= (double)tune().small_tail_to) {
                    hipLaunchKernelGGL((conv_igemm_kernel<T, MODE, 2, 2, 1, 1, BK_SMALL, true, EDL_PF_SMALL_TAIL>), grid, dim3(256), 0, st, a);
                    break;
                }
            }
            hipLaunchKernelGGL((conv_igemm_kernel<T, MODE, 2, 2, 1, 1, BK_SMALL, true, PF_SMALL>), grid, dim3(256), 0, st, a);
            break;
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


static bool conv_fast(int dtype, int mode, const ConvArgs& a) {
    const int ovec = (mode == CONV_WGRAD || dtype != 1) ? 4 : 8;
    return a.vecA && a.vecB && a.Nn % ovec == 0;
}

// every multiply-shift division of the vector kernel is exact for this problem
static bool conv_magic_ok(int mode, const ConvArgs& a) {
    if (mode == CONV_WGRAD) return true;
    const int inner = mode == CONV_FWD ? a.C : a.K, taps = mode == CONV_FWD ? a.S : a.ns;
    const int pix = mode == CONV_FWD ? a.Ho * a.Wo : a.Hc * a.Wc, wpix = mode == CONV_FWD ? a.Wo : a.Wc;
    const double kmax = (double)a.Kred + 256.0, mmax = (double)a.M + 256.0;
    return magic_fits(kmax, inner) && magic_fits(kmax / (inner > 0 ? inner : 1) + 1.0, taps) &&
           magic_fits(mmax, pix) && magic_fits((double)pix, wpix);
}

template <int MODE>
static void launch_mode(int dtype, TileCfg t, dim3 grid, const ConvArgs& a_in, hipStream_t st) {
    ConvArgs a = a_in;
    if (MODE == CONV_FWD) { a.magic_inner = magic_of(a.C); a.magic_taps = magic_of(a.S); }
    else if (MODE == CONV_DGRAD) { a.magic_inner = magic_of(a.K); a.magic_taps = magic_of(a.ns); }
    if (MODE == CONV_FWD) { a.magic_hw = magic_of(a.Ho * a.Wo); a.magic_w = magic_of(a.Wo); }
    else if (MODE == CONV_DGRAD) { a.magic_hw = magic_of(a.Hc * a.Wc); a.magic_w = magic_of(a.Wc); }
    a.stride_shift = a.stride >= 4 ? 2 : a.stride >= 2 ? 1 : 0;
    const bool magic_ok = conv_magic_ok(MODE, a);
    const bool fast = conv_fast(dtype, MODE, a) && magic_ok;
    if (!fast) {
        t = T64x64;
        grid.x = (a.M + 63) / 64;
        grid.y = (a.Nn + 63) / 64;
    }
    // Tile order: the reduction cuts are the slowest index, so a die's run of tiles
    // stays within few cuts; inside a cut the tiles that share the larger operand
    // (activations: the same row tile; weights: the same column tile) are neighbours.
    const int tune_xcd = (int)tune().xcd, tune_order = (int)tune().order;
    a.xcd_chunked = tune_xcd;
    if (tune_order >= 0) a.n_fastest = tune_order;
    else if (MODE == CONV_WGRAD) a.n_fastest = 1;
    else a.n_fastest = (double)a.M * (MODE == CONV_FWD ? a.C : a.K) >= (double)a.Nn * a.Kred;
    // algorithmic work: 2*M*N*K flops; operands and result touched once
    const double esz = dtype == 1 ? 2.0 : 4.0;
    const double flops = 2.0 * (double)a.M * a.Nn * a.Kred;
    double bytes;
    if (MODE == CONV_FWD) bytes = esz * ((double)a.N * a.H * a.W * a.C + (double)a.Nn * a.Kred) + (a.out_fp32 ? 4.0 : esz) * (double)a.M * a.Nn;
    else if (MODE == CONV_DGRAD) {
        // dy, weights, dx; plus what a fused epilogue reads at every output position: the gradient already
        // there, the activation that masks it, the batch norm's input for the second sum
        const double extra = (a.accumulate ? 1.0 : 0.0) + (a.mask_act ? 1.0 : 0.0) + (a.xin ? 1.0 : 0.0);
        bytes = esz * ((double)a.N * a.Ho * a.Wo * a.K + (double)a.Nn * a.Kred + (1.0 + extra) * (double)a.M * a.Nn);
    } else bytes = esz * ((double)a.Kred * a.K + (double)a.N * a.H * a.W * a.C) + 4.0 * (double)a.M * a.Nn;
    const char* label = conv_label(dtype, MODE, t);
    static const bool by_shape = getenv("EDL_PROFILE_BY_SHAPE") != nullptr;
    if (by_shape && prof_enabled()) {
        // one profile line per distinct problem shape instead of per kernel family
        static std::deque<std::string> names;
        char buf[160];
        snprintf(buf, sizeof(buf), "%s M=%d N=%d K=%d r%d s%d grid=%ux%ux%u", label, a.M, a.Nn, a.Kred, a.R, a.stride, grid.x, grid.y, grid.z);
        const char* found = nullptr;
        for (const std::string& n : names) if (n == buf) { found = n.c_str(); break; }
        if (!found) { names.emplace_back(buf); found = names.back().c_str(); }
        label = found;
    }
    ProfScope ps(label, flops, bytes, st);
    if (dtype == 1) launch_cfg<bf16_t, MODE>(t, fast, grid, a, st);
    else launch_cfg<float, MODE>(t, fast, grid, a, st);
}

static ConvArgs base_args(const ConvGeom& g) {
    ConvArgs a = {};
    a.N = g.N; a.H = g.H; a.W = g.W; a.C = g.C; a.K = g.K; a.R = g.R; a.S = g.S;
    a.stride = g.stride; a.pad = g.pad; a.Ho = g.Ho; a.Wo = g.Wo;
    a.ph = a.pw = a.r0 = a.s0 = 0; a.nr = g.R; a.ns = g.S; a.Hc = g.H; a.Wc = g.W;
    a.red_stride = kRedRowBlocks;
    return a;
}

// Partial column sums of a launch with more row tiles than the reduction scratch has room for:
// out[r][j] = sum of wide[r][j*group .. (j+1)*group), in order; r = (sum kind, channel).
__global__ __launch_bounds__(256) void compact_sums_kernel(const float* __restrict__ wide, int tiles, int group, int out_tiles,
                                                           float* __restrict__ out) {
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    const int r = blockIdx.y;
    if (j >= out_tiles) return;
    const float* src = wide + (int64_t)r * tiles;
    int e = (j + 1) * group;
    if (e > tiles) e = tiles;
    float s = 0.f;
    for (int i = j * group; i < e; ++i) s += src[i];
    out[(int64_t)r * kRedRowBlocks + j] = s;
}

// Where an epilogue leaves its column sums: the reduction scratch itself if the row tiles fit it, else the wide
// buffer (compacted afterwards by finish_sums), else nowhere (nullptr: the separate reduction kernel runs).
static float* sums_target(float* sums, const WideSums& wide, int row_tiles, int channels, int* stride) {
    *stride = kRedRowBlocks;
    if (sums == nullptr || row_tiles <= kRedRowBlocks) return sums;
    if (wide.buf == nullptr || wide.floats < (size_t)2 * channels * row_tiles) return nullptr;
    *stride = row_tiles;
    return wide.buf;
}

// Returns the number of partial sums per channel now in `sums`.
static int finish_sums(float* sums, const WideSums& wide, int row_tiles, int channels, hipStream_t st) {
    if (row_tiles <= kRedRowBlocks) return row_tiles;
    const int group = (row_tiles + kRedRowBlocks - 1) / kRedRowBlocks;
    const int out_tiles = (row_tiles + group - 1) / group;
    ProfScope ps("compact_sums", 0.0, 4.0 * 2.0 * channels * ((double)row_tiles + out_tiles), st);
    hipLaunchKernelGGL(compact_sums_kernel, dim3((out_tiles + 255) / 256, 2 * channels), dim3(256), 0, st, wide.buf, row_tiles, group,
                       out_tiles, sums);
    return out_tiles;
}

size_t conv_wide_sums_floats(int dtype, const ConvGeom& g) {
    (void)dtype;
    // the narrowest row tile is 64 rows
    const int64_t fwd_tiles = ((int64_t)g.N * g.Ho * g.Wo + 63) / 64, dgrad_tiles = ((int64_t)g.N * g.H * g.W + 63) / 64;
    size_t need = 0;
    if (fwd_tiles > kRedRowBlocks) need = std::max(need, (size_t)(2 * fwd_tiles * g.K));
    if (dgrad_tiles > kRedRowBlocks && g.stride == 1) need = std::max(need, (size_t)(2 * dgrad_tiles * g.C));
    return need;
}

// Cut of the reduction for forward / dgrad problems that give too few tiles to
// fill the chip but have a long reduction (late stages at small batch, fully
// connected layers): returns the number of splits (1 = none).  The target is little more than one
// workgroup per CU: every further cut costs the finishing kernel more partial sums than the fuller chip
// gains (measured on ResNet-50 at a shard of 32: 768 -> 320 workgroups, 4.73 -> 4.69 ms per step;
// VGG-16 5.20 -> 5.14 ms).
static int plan_splitk(int dtype, int M, int Nn, int Kred, int bm, int bn, int* ksplit) {
    const int BK = dtype == 1 ? 64 : 32;
    const int64_t tiles = (int64_t)((M + bm - 1) / bm) * ((Nn + bn - 1) / bn);
    const int nk = (Kred + BK - 1) / BK;
    int splits = 1;
    const int max_tiles = (int)tune().splitk_tiles, target = (int)tune().splitk_target;
    if (tiles < max_tiles && nk >= 8) {
        splits = (int)((target + tiles - 1) / tiles);
        if (splits > nk / 4) splits = nk / 4;
        if (splits > 8) splits = 8;
        if (splits < 1) splits = 1;
    }
    int ks = (nk + splits - 1) / splits * BK;
    *ksplit = ks;
    return (Kred + ks - 1) / ks;
}

// Returns the number of row blocks whose column sums it left in stats (0 if stats is null).
template <typename T>
static int launch_finish(const ConvArgs& a, int splits, float* stats, hipStream_t st, const DgradMask* mask = nullptr) {
    const int col_blocks = (a.Nn + 63) / 64;
    // about 1024 workgroups, at least 16 rows each
    int64_t rb = (1024 + col_blocks - 1) / col_blocks;
    const int64_t max_rb = ((int64_t)a.M + 15) / 16;
    if (rb > max_rb) rb = max_rb;
    if (rb > kRedRowBlocks) rb = kRedRowBlocks;
    if (rb < 1) rb = 1;
    const int rows_per_block = (int)(((int64_t)a.M + rb - 1) / rb);
    const int row_blocks = (int)(((int64_t)a.M + rows_per_block - 1) / rows_per_block);
    ProfScope ps("splitk_finish", 0.0, 4.0 * (double)a.M * a.Nn * splits + (a.out_fp32 ? 4.0 : (double)sizeof(T)) * (double)a.M * a.Nn, st);
    if (mask != nullptr)
        hipLaunchKernelGGL((splitk_finish_kernel<T, true>), dim3(col_blocks, row_blocks), dim3(256), 0, st, a.partial, a.out, a.bias,
                           (int64_t)a.M, a.Nn, splits, a.relu, a.out_fp32, a.accumulate, rows_per_block, stats,
                           (const T*)mask->act, (const T*)mask->xin, mask->mean_rstd, a.acc_src);
    else
        hipLaunchKernelGGL((splitk_finish_kernel<T, false>), dim3(col_blocks, row_blocks), dim3(256), 0, st, a.partial, a.out, a.bias,
                           (int64_t)a.M, a.Nn, splits, a.relu, a.out_fp32, a.accumulate, rows_per_block, stats,
                           (const T*)nullptr, (const T*)nullptr, (const float*)nullptr, a.acc_src);
    return stats ? row_blocks : 0;
}

size_t conv_splitk_scratch_bytes(int dtype, const ConvGeom& g) {
    size_t need = 0;
    for (int mode = 0; mode < 2; ++mode) {
        if (mode == 1 && g.stride != 1) continue;
        const int M = mode == 0 ? g.N * g.Ho * g.Wo : g.N * g.H * g.W;
        const int Nn = mode == 0 ? g.K : g.C;
        const int Kred = mode == 0 ? g.R * g.S * g.C : g.R * g.S * g.K;
        int bm, bn, ks;
        pick_tile(M, Nn, Kred, &bm, &bn, mode == 0 && Kred <= 128);
        const int splits = plan_splitk(dtype, M, Nn, Kred, bm, bn, &ks);
        if (splits > 1) need = std::max(need, (size_t)splits * M * Nn * sizeof(float));
    }
    return need;
}

int launch_conv_fwd(int dtype, const ConvGeom& g, const void* x, const void* w, const float* bias, bool relu,
                    bool out_fp32, void* y, float* scratch, size_t scratch_bytes, float* stats, WideSums wide, hipStream_t st) {
    const int VEC = dtype == 1 ? 8 : 4;
    ConvArgs a = base_args(g);
    a.A = x; a.B = w; a.out = y; a.bias = bias;
    a.M = g.N * g.Ho * g.Wo; a.Nn = g.K; a.Kred = g.R * g.S * g.C;
    a.relu = relu; a.out_fp32 = out_fp32;
    const double esz = dtype == 1 ? 2.0 : 4.0;
    const double bA = esz * (double)g.N * g.H * g.W * g.C, bB = esz * (double)a.Nn * a.Kred;
    a.vecA = (g.C % VEC == 0) && bA < 2147483648.0; a.vecB = (a.Kred % VEC == 0) && bB < 2147483648.0;
    a.bytesA = a.vecA ? (unsigned)bA : 0; a.bytesB = a.vecB ? (unsigned)bB : 0;
    a.ksplit = a.Kred;
    a.ldb = a.Kred;
    int bm, bn;
    const TileCfg t = pick_tile(a.M, a.Nn, a.Kred, &bm, &bn, a.Kred <= 128);
    int splits = 1, ks = a.Kred;
    if (conv_fast(dtype, CONV_FWD, a)) {
        splits = plan_splitk(dtype, a.M, a.Nn, a.Kred, bm, bn, &ks);
        if (splits > 1 && (scratch == nullptr || scratch_bytes < (size_t)splits * a.M * a.Nn * sizeof(float))) splits = 1;
    }
    if (splits > 1) { a.ksplit = ks; a.partial = scratch; }
    const int row_tiles = (a.M + bm - 1) / bm;
    const bool tune_stats = tune().fused_stats != 0;
    const bool want_stats = tune_stats && stats != nullptr && !out_fp32 && conv_fast(dtype, CONV_FWD, a) && conv_magic_ok(CONV_FWD, a);
    // whole reduction in one workgroup: the epilogue leaves the sums; cut reduction: the finishing kernel does
    float* const target = (want_stats && splits == 1) ? sums_target(stats, wide, row_tiles, a.Nn, &a.red_stride) : nullptr;
    const bool fused = target != nullptr;
    a.stats = target;
    launch_mode<CONV_FWD>(dtype, t, dim3(row_tiles, (a.Nn + bn - 1) / bn, splits), a, st);
    if (splits > 1) {
        float* fs = want_stats ? stats : nullptr;
        return dtype == 1 ? launch_finish<bf16_t>(a, splits, fs, st) : launch_finish<float>(a, splits, fs, st);
    }
    return fused ? finish_sums(stats, wide, row_tiles, a.Nn, st) : 0;
}

int launch_conv_dgrad(int dtype, const ConvGeom& g, const void* dy, const void* wT, bool accumulate, void* dx,
                      float* scratch, size_t scratch_bytes, const DgradMask* mask, hipStream_t st, const void* acc_src) {
    int fused_rows = 0;
    const int VEC = dtype == 1 ? 8 : 4;
    ConvArgs a = base_args(g);
    a.A = dy; a.B = wT; a.out = dx;
    a.Nn = g.C;
    a.ldb = g.R * g.S * g.K;
    a.accumulate = accumulate;
    a.acc_src = (accumulate && g.stride == 1) ? acc_src : nullptr;
    const double esz = dtype == 1 ? 2.0 : 4.0;
    const double bA = esz * (double)g.N * g.Ho * g.Wo * g.K, bB = esz * (double)a.Nn * a.ldb;
    // the vector gather of dy divides pixel coordinates by the stride with a shift
    const bool stride_pow2 = g.stride == 1 || g.stride == 2 || g.stride == 4;
    a.vecA = (g.K % VEC == 0) && bA < 2147483648.0 && stride_pow2; a.vecB = (a.ldb % VEC == 0) && bB < 2147483648.0;
    a.bytesA = a.vecA ? (unsigned)bA : 0; a.bytesB = a.vecB ? (unsigned)bB : 0;
    // one launch per residue class of the input pixel modulo the stride
    for (int ph = 0; ph < g.stride && ph < g.H; ++ph) {
        for (int pw = 0; pw < g.stride && pw < g.W; ++pw) {
            a.ph = ph; a.pw = pw;
            a.Hc = (g.H - ph + g.stride - 1) / g.stride;
            a.Wc = (g.W - pw + g.stride - 1) / g.stride;
            a.r0 = (ph + g.pad) % g.stride;
            a.s0 = (pw + g.pad) % g.stride;
            a.nr = a.r0 < g.R ? (g.R - a.r0 + g.stride - 1) / g.stride : 0;
            a.ns = a.s0 < g.S ? (g.S - a.s0 + g.stride - 1) / g.stride : 0;
            a.M = g.N * a.Hc * a.Wc;
            a.Kred = a.nr * a.ns * g.K;
            a.ksplit = a.Kred > 0 ? a.Kred : 1;
            a.partial = nullptr;
            if (a.Kred == 0 && accumulate) continue;      // nothing reaches these pixels
            int bm, bn;
            // an epilogue that adds to the gradient already there, masks and sums it reads three more tensors
            // than it writes: 128x64 tiles (twice the workgroups, half the vectors in flight per lane; measured
            // -0.4% of the ResNet-50 step, 64x64 tiles +1.5%)
            const int join_tile = (int)tune().join_tile;
            const bool heavy = join_tile != 0 && mask != nullptr && mask->act != nullptr && accumulate && g.stride == 1;
            const TileCfg t = pick_tile(a.M, a.Nn, a.Kred, &bm, &bn, heavy);
            int splits = 1, ks = a.ksplit;
            if (g.stride == 1 && conv_fast(dtype, CONV_DGRAD, a)) {
                splits = plan_splitk(dtype, a.M, a.Nn, a.Kred, bm, bn, &ks);
                if (splits > 1 && (scratch == nullptr || scratch_bytes < (size_t)splits * a.M * a.Nn * sizeof(float))) splits = 1;
            }
            if (splits > 1) { a.ksplit = ks; a.partial = scratch; }
            const int row_tiles = (a.M + bm - 1) / bm;
            // masked store and column sums in the epilogue: one launch that covers every pixel and leaves the
            // final gradient (it may add to what other readers of the tensor have left there)
            const bool tune_mask = tune().fused_mask != 0;
            float* target = nullptr;
            if (tune_mask && mask != nullptr && mask->act != nullptr && g.stride == 1 && splits == 1 &&
                conv_fast(dtype, CONV_DGRAD, a) && conv_magic_ok(CONV_DGRAD, a))
                target = sums_target(mask->sums, mask->wide, row_tiles, a.Nn, &a.red_stride);
            const bool fuse = target != nullptr;
            a.mask_act = fuse ? mask->act : nullptr;
            a.xin = fuse ? mask->xin : nullptr;
            a.mean_rstd = fuse ? mask->mean_rstd : nullptr;
            a.msum = target;
            launch_mode<CONV_DGRAD>(dtype, t, dim3(row_tiles, (a.Nn + bn - 1) / bn, splits), a, st);
            if (fuse) fused_rows = finish_sums(mask->sums, mask->wide, row_tiles, a.Nn, st);
            if (splits > 1) {
                // a cut reduction: the finishing kernel masks and sums instead of the epilogue
                const bool tune_cut = tune().fused_mask_cut != 0;
                const bool cut_mask = tune_cut && tune_mask && mask != nullptr && mask->act != nullptr && mask->sums != nullptr &&
                                      g.stride == 1 && a.Nn % 4 == 0;
                const DgradMask* fm = cut_mask ? mask : nullptr;
                float* fs = cut_mask ? mask->sums : nullptr;
                fused_rows = dtype == 1 ? launch_finish<bf16_t>(a, splits, fs, st, fm) : launch_finish<float>(a, splits, fs, st, fm);
            }
        }
    }
    return fused_rows;
}

struct WgradPlan {
    TileCfg t;
    int bm, bn, splits, ksplit;
    int64_t tiles;
};

// Tile and split of the weight gradient.  Its output is small and its
// reduction (the pixels) long, so parallelism comes from cutting the reduction;
// every split costs a float32 partial tile that is written and read again, so
// layers whose output already gives enough tiles are split little or not at all.
static WgradPlan plan_wgrad(const ConvGeom& g) {
    WgradPlan p;
    const int M = g.K, Nn = g.R * g.S * g.C, Kred = g.N * g.Ho * g.Wo;
    const int64_t t128 = (int64_t)((M + 127) / 128) * ((Nn + 127) / 128);
    const int64_t t64 = (int64_t)((M + 63) / 64) * ((Nn + 63) / 64);
    if (Nn <= 32) p.t = T128x32;
    else if (M <= 64 || Nn <= 64) p.t = (Nn <= 64 && M >= 128) ? T128x64 : T64x64;
    else if (t128 >= 128) p.t = T128x128;
    else if (t64 >= 256 && Kred < 4096) p.t = T64x64;   // long reductions are cut instead (below)
    else p.t = T128x128;
    switch (p.t) {
        case T128x128: p.bm = 128; p.bn = 128; break;
        case T128x64: p.bm = 128; p.bn = 64; break;
        case T128x32: p.bm = 128; p.bn = 32; break;
        default: p.bm = 64; p.bn = 64; break;
    }
    p.tiles = (int64_t)((M + p.bm - 1) / p.bm) * ((Nn + p.bn - 1) / p.bn);
    // The weight gradients run beside the input-gradient chain on a second stream: about one workgroup per
    // two CUs leaves that chain the room it needs (ResNet-50 at a shard of 32: 256 -> 128 workgroups, alone on
    // the chip 3% slower per step, beside the main stream 1.4% faster; ResNet-152 1.8%; below 96 the second
    // stream becomes the longer one).
    const int target = (int)tune().wgrad_blocks;
    int64_t splits = (target + p.tiles - 1) / p.tiles;
    // A long reduction (VGG-16's layers on large images at a shard of 32) is cut into two workgroups per CU
    // (all that are resident at once), as long as each cut keeps long_ks elements: the partial results are
    // small beside the operands there, and a second workgroup hides the operand latency that one per CU
    // leaves exposed.  Measured on VGG-16: 5.28 -> 5.14 ms per step; three per CU (a second, ragged round
    // of workgroups) is slower again.
    const int long_target = (int)tune().wgrad_long_blocks, long_ks = (int)tune().wgrad_long_ks;
    const int64_t more = std::min<int64_t>(long_target / p.tiles, Kred / (long_ks > 0 ? long_ks : 1));
    if (more > splits) splits = more;
    const int64_t max_splits = (Kred + 255) / 256;  // at least 4 reduction steps per split
    if (splits > max_splits) splits = max_splits;
    if (splits < 1) splits = 1;
    int64_t ks = (Kred + splits - 1) / splits;
    ks = (ks + 63) / 64 * 64;
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
    const double esz = dtype == 1 ? 2.0 : 4.0;
    const double bA = esz * (double)a.Kred * g.K, bB = esz * (double)g.N * g.H * g.W * g.C;
    a.vecA = (g.K % VEC == 0) && bA < 2147483648.0; a.vecB = (g.C % VEC == 0) && bB < 2147483648.0;
    a.bytesA = a.vecA ? (unsigned)bA : 0; a.bytesB = a.vecB ? (unsigned)bB : 0;
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
        ProfScope ps("wgrad_reduce", 0.0, 4.0 * (double)n * (p.splits + 1), st);
        // dw may sit at any float offset of the flat gradient vector: vectors only if it is 16-byte aligned
        if (n % 4 == 0 && ((uintptr_t)dw & 15) == 0) {
            int64_t blocks = (n / 4 + 255) / 256;
            if (blocks > 8192) blocks = 8192;
            hipLaunchKernelGGL(wgrad_reduce_kernel<4>, dim3((int)blocks), dim3(256), 0, st, scratch, dw, n, p.splits);
        } else {
            int64_t blocks = (n + 255) / 256;
            if (blocks > 8192) blocks = 8192;
            hipLaunchKernelGGL(wgrad_reduce_kernel<1>, dim3((int)blocks), dim3(256), 0, st, scratch, dw, n, p.splits);
        }
    }
}

}  // namespace edl
