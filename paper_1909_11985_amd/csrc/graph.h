// Model tables: a static list of layer operations over numbered activation
// tensors, plus the layout of the flat parameter vector.  Host only.
#pragma once
#include <cstdint>
#include <string>
#include <vector>

#include "../../include/edl.h"

namespace edl {

enum OpKind { OP_CONV, OP_BN, OP_MAXPOOL, OP_GAVGPOOL, OP_LOSS };

struct Tensor {
    int H = 0, W = 0, C = 0;      // per-sample shape, channels innermost
    int alias_of = -1;            // a flattened view shares its source's storage
    bool fp32 = false;            // the logits stay float32 in every configuration
    int64_t elems() const { return (int64_t)H * W * C; }
};

struct Op {
    OpKind kind;
    int x = -1, y = -1, res = -1;          // input, output, residual input (batch norm only)
    int K = 0, R = 1, S = 1, stride = 1, pad = 0;
    bool bias = false, relu = false;
    int64_t w_off = -1, b_off = -1;        // conv weight / bias, or batch-norm scale / shift
    int64_t run_off = -1;                  // batch-norm running mean, then variance
    std::string name;
};

struct ParamTensor {
    std::string name;
    int64_t off, size, fan_in;             // fan_in = 0: not drawn at random
    bool is_gamma;
};

struct Graph {
    std::vector<Tensor> tensors;           // tensor 0 is the input image
    std::vector<Op> ops;
    std::vector<ParamTensor> params;
    int64_t P = 0, R = 0;
    int logits = -1;
    int classes = 0;

    int add_tensor(int H, int W, int C);
    int conv(int x, int K, int R, int stride, int pad, bool bias, bool relu, const std::string& name);
    int bn(int x, bool relu, int res, const std::string& name);
    int maxpool(int x, int k, int stride, int pad);
    int gavgpool(int x);
    int flatten(int x);
    void loss(int x);
    double flops_per_sample() const;
};

// Fills g for the configuration; returns EDL_OK or EDL_EINVAL (message via set_error).
int build_graph(const edl_config& cfg, Graph& g);

// Host integer / initialisation logic
uint64_t splitmix64_at(uint64_t key, uint64_t j);
void epoch_permutation(uint64_t seed, int64_t epoch, int64_t N, std::vector<int64_t>& perm);
void he_init(const Graph& g, uint64_t seed, float* out);

void set_error(const char* fmt, ...);
const char* get_error();

}  // namespace edl
