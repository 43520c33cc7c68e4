// Host-callable launchers of the HIP kernels.  `dtype` is EDL_DTYPE_*: the
// element type of activation tensors and of the weight copies the matrix
// cores read.  Every launcher only queues work on `st`.
#pragma once
#include <hip/hip_runtime.h>
#include <cstddef>
#include <cstdint>

namespace edl {

constexpr int kMaxP = 16;           // gradient buffers one update launch can average
constexpr int kRedRowBlocks = 1024;   // upper bound of row blocks in column reductions

struct GradPtrs { const float* g[kMaxP]; };
struct ShardShares { float share[kMaxP]; };   // a shard's part of the mini-batch

// ---- aggregation + update, copies ----------------------------------------
// max_blocks > 0 holds the launch to that many workgroups (a pass that runs in the background of other work).
void launch_average_update(int p, const GradPtrs& grads, float* w, float* v, uint16_t* w16, int64_t P,
                           float lr, float momentum, float wd, hipStream_t st, int max_blocks = 0);
// aggregate = sum_k shares[k] * grads[k] (shards of unequal size)
void launch_weighted_update(int np, const GradPtrs& grads, const ShardShares& shares, float* w, float* v, uint16_t* w16,
                            int64_t P, float lr, float momentum, float wd, hipStream_t st);
// Adam on the aggregated gradient.  shares == nullptr: the mean of the p gradients; otherwise sum_k shares->share[k]*G_k.
// c1 = 1/(1-beta1^t), c2 = 1/(1-beta2^t).
void launch_adam_update(int p, const GradPtrs& grads, const ShardShares* shares, float* w, float* m, float* s, uint16_t* w16,
                        int64_t P, float lr, float beta1, float beta2, float eps, float wd, float c1, float c2, hipStream_t st,
                        int max_blocks = 0);
void launch_copy(void* dst, const void* src, size_t bytes, hipStream_t st);
void launch_fill_f32(float* dst, float value, int64_t n, hipStream_t st);
// dst[c][r][s][k] = cast(src[k][r][s][c]) (weights for the input-gradient contraction) for every
// layer of a model in one launch, from a table in device memory
struct TransposeEntry {
    int64_t src_off;     // floats from the start of the parameter vector
    int64_t dst_off;     // bytes from the start of the arena
    int K, RS, C;
    int tile_start;      // index of the layer's first 32x32 tile among all layers' tiles
};
void launch_weight_transpose_all(int dtype, const float* w, void* arena, const TransposeEntry* dev_table, int entries,
                                 int total_tiles, double bytes, hipStream_t st);
// bf16 layers with K and C multiples of 8, from the bf16 copy of the weights; tile_start counts 64x64 tiles
void launch_weight_transpose_bf16(const uint16_t* w16, void* arena, const TransposeEntry* dev_table, int entries,
                                  int total_tiles, double bytes, hipStream_t st);
// dst = cast(src) for float32 -> bf16 (weight copy after restore / set_params)
void launch_cast_bf16(const float* src, uint16_t* dst, int64_t n, hipStream_t st);

// ---- input --------------------------------------------------------------
void launch_gather(int dtype, const float* data_x, const int32_t* data_y, const int64_t* idx, int n,
                   int64_t sample_elems, void* out_x, int32_t* out_y, hipStream_t st);

// images with C channels written as pixels of one zero-padded 16-byte vector each
void launch_gather_pad(int dtype, const float* data_x, const int32_t* data_y, const int64_t* idx, int n, int64_t pixels,
                       int C, void* out_x, int32_t* out_y, hipStream_t st);
// weights [rows][C] float32 -> [rows][Cp] dtype, zero padded; and the way back for their gradient
void launch_pad_weights(int dtype, const float* src, void* dst, int64_t rows, int C, int Cp, hipStream_t st);
void launch_unpad_rows(const float* src, float* dst, int64_t rows, int C, int Cp, hipStream_t st);

// ---- implicit-GEMM convolution --------------------------------------------
enum ConvMode { CONV_FWD = 0, CONV_DGRAD = 1, CONV_WGRAD = 2 };

struct ConvGeom {
    int N, H, W, C;          // input images
    int K, R, S, stride, pad, Ho, Wo;
};

// y = conv(x, w) (+bias) (ReLU); y is float32 if out_fp32 else dtype.
// stats (may be null): the batch-norm reduction's partial-sum scratch.  If the launch can, it also leaves
// there the per-row-tile column sums of y and y*y and returns the number of row tiles (what
// launch_bn_forward takes as stats_row_blocks); it returns 0 if it left none.
// Partial column sums of launches with more than kRedRowBlocks row tiles are written into `wide`
// (2 * channels * row tiles floats, if it is large enough) and summed in groups into the standard scratch.
struct WideSums { float* buf; size_t floats; };
int launch_conv_fwd(int dtype, const ConvGeom& g, const void* x, const void* w, const float* bias, bool relu,
                    bool out_fp32, void* y, float* scratch, size_t scratch_bytes, float* stats, WideSums wide, hipStream_t st);
// floats `wide` must hold for this layer's forward statistics and input-gradient sums (0 if never needed)
size_t conv_wide_sums_floats(int dtype, const ConvGeom& g);
// What the layer that produced the convolution's input wants from the gradient dx when it ends in a ReLU:
// dx * (act > 0), and per-channel sums of that over the rows (plain, and times (xin - mean) * rstd if xin is
// given: a batch norm's backward sums).  sums: the column-reduction partial-sum scratch.
struct DgradMask {
    const void* act;          // the producer's output (= this convolution's input), dtype elements
    const void* xin;          // the producing batch norm's input, or null
    const float* mean_rstd;   // with xin: mean[C], rstd[C]
    float* sums;
    WideSums wide;
};
// dx (+)= conv^T(dy, wT); wT is the [C][R][S][K] copy.  mask (may be null): if the launch can (stride 1, one
// launch over all pixels, writing), dx is stored already masked and the sums are left in mask->sums; returns
// the number of row tiles summed (what the producer's backward takes as its row-block count), else 0 and dx
// is the plain gradient.
// acc_src (stride 1 with accumulate only; may be null): the gradient that is added to is read from this tensor of
// dx's shape instead of from dx itself (dx is then written, not read).
int launch_conv_dgrad(int dtype, const ConvGeom& g, const void* dy, const void* wT, bool accumulate, void* dx,
                      float* scratch, size_t scratch_bytes, const DgradMask* mask, hipStream_t st,
                      const void* acc_src = nullptr);
// float32 scratch a forward / dgrad launch may use to cut a long reduction of a small problem
size_t conv_splitk_scratch_bytes(int dtype, const ConvGeom& g);
// dw = x^T * dy, float32 [K][R][S][C]; scratch holds split partial sums
void launch_conv_wgrad(int dtype, const ConvGeom& g, const void* x, const void* dy, float* dw, float* scratch,
                       size_t scratch_bytes, hipStream_t st);
size_t conv_wgrad_scratch_bytes(const ConvGeom& g);

// ---- batch norm, bias / ReLU backward --------------------------------------
// partial: float32 scratch of 2 * kRedRowBlocks * C floats
void launch_bn_forward(int dtype, const void* x, const void* res, void* y, const float* gamma, const float* beta,
                       float* save_mean_rstd /*[2C]*/, float* running /*[2C] or null*/, int64_t M, int C,
                       bool relu, float* partial, int stats_row_blocks /*> 0: partial already holds the sums*/,
                       hipStream_t st);
// sums_row_blocks > 0: partial already holds the two backward sums over that many row blocks (left there by
// the dgrad that produced dy, which is then also masked already)
void launch_bn_backward(int dtype, const void* x, const void* y, const void* dy, void* dx, void* dres,
                        bool dres_accumulate, const float* gamma, const float* save_mean_rstd,
                        float* dgamma, float* dbeta, int64_t M, int C, bool relu, float* partial, float* coef /*[2C]*/,
                        int sums_row_blocks, hipStream_t st);
// dy <- dy * (y > 0) in place if relu; dbias[c] = sum_rows dy (if dbias).
// sums_row_blocks > 0: dy is masked already and partial holds its column sums over that many row blocks.
void launch_bias_relu_backward(int dtype, const void* y, void* dy, float* dbias, int64_t M, int C, bool relu,
                               float* partial, int sums_row_blocks, hipStream_t st);

// ---- pooling --------------------------------------------------------------
void launch_maxpool_forward(int dtype, const void* x, void* y, uint8_t* arg, int N, int H, int W, int C, int k,
                            int stride, int pad, int Ho, int Wo, hipStream_t st);
// relu_act: if the pooled tensor is the output of a ReLU layer with no other reader, that output; the gradient is
// then stored multiplied by (relu_act > 0) where the kernel taken supports it.  Returns whether it was.
bool launch_maxpool_backward(int dtype, const void* dy, const uint8_t* arg, void* dx, bool accumulate, int N, int H,
                             int W, int C, int k, int stride, int pad, int Ho, int Wo, const void* relu_act, hipStream_t st);
void launch_gavgpool_forward(int dtype, const void* x, void* y, int N, int HW, int C, hipStream_t st);
void launch_gavgpool_backward(int dtype, const void* dy, void* dx, bool accumulate, int N, int HW, int C,
                              hipStream_t st);

// ---- loss -------------------------------------------------------------------
// logits float32 [n][C]; dlogits in dtype; loss_out[0] = mean over the n rows
void launch_softmax_ce(int dtype, const float* logits, const int32_t* labels, void* dlogits, float* row_loss,
                       float* loss_out, int n, int C, hipStream_t st);

// register-resident MFMA loop (attainable matrix rate); returns the flops the launch issues
double launch_mfma_rate(int dtype, int blocks, int iters, float* sink, hipStream_t st);

}  // namespace edl
