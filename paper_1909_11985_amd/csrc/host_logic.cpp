// Host-side integer logic and model tables: shard assignment (sections 3.1
// and 4.3 of the paper), He initialisation, and the layer lists of the four
// model families.  No GPU code here.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <thread>

#include "graph.h"

namespace edl {

// ---------------------------------------------------------------- errors
static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}
const char* get_error() { return g_err; }

// ---------------------------------------------------------------- generator
// SplitMix64 used as a counter-based generator: draw j of a stream is the
// finaliser applied to key + (j+1)*golden.
static const uint64_t kGolden = 0x9E3779B97F4A7C15ull;
static const uint64_t kInitKey = 0xD1B54A32D192ED03ull;

uint64_t splitmix64_at(uint64_t key, uint64_t j) {
    uint64_t z = key + (j + 1) * kGolden;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// The leader's random permutation of section 4.3, one per epoch: Fisher-Yates
// from the last position down, partner index = high 64 bits of draw*(i+1).
void epoch_permutation(uint64_t seed, int64_t epoch, int64_t N, std::vector<int64_t>& perm) {
    const uint64_t key = seed ^ (kGolden * (uint64_t)(epoch + 1));
    perm.resize((size_t)N);
    for (int64_t i = 0; i < N; ++i) perm[(size_t)i] = i;
    uint64_t draw = 0;
    for (int64_t i = N - 1; i >= 1; --i) {
        const uint64_t r = splitmix64_at(key, draw++);
        const uint64_t j = (uint64_t)(((unsigned __int128)r * (unsigned __int128)(uint64_t)(i + 1)) >> 64);
        const int64_t t = perm[(size_t)i];
        perm[(size_t)i] = perm[(size_t)j];
        perm[(size_t)j] = t;
    }
}

// He-normal weights by Box-Muller on the counter-based draws, one stream per
// parameter tensor (keyed by the tensor's position in the flat vector).
void he_init(const Graph& g, uint64_t seed, float* out) {
    for (size_t t = 0; t < g.params.size(); ++t) {
        const ParamTensor& pt = g.params[t];
        float* dst = out + pt.off;
        if (pt.fan_in == 0) {
            const float fill = pt.is_gamma ? 1.0f : 0.0f;
            for (int64_t i = 0; i < pt.size; ++i) dst[i] = fill;
            continue;
        }
        const uint64_t key = seed ^ (kInitKey * (uint64_t)(t + 1));
        const double sd = std::sqrt(2.0 / (double)pt.fan_in);
        const double two_pi = 2.0 * 3.14159265358979323846;
        const int64_t pairs = (pt.size + 1) / 2;
        const int64_t size = pt.size;
        auto fill = [=](int64_t q0, int64_t q1) {
            for (int64_t q = q0; q < q1; ++q) {
                const uint64_t r1 = splitmix64_at(key, (uint64_t)(2 * q));
                const uint64_t r2 = splitmix64_at(key, (uint64_t)(2 * q + 1));
                const double u1 = ((double)(r1 >> 11) + 1.0) * 0x1.0p-53;
                const double u2 = (double)(r2 >> 11) * 0x1.0p-53;
                const double rad = std::sqrt(-2.0 * std::log(u1));
                const double ang = two_pi * u2;
                dst[2 * q] = (float)(rad * std::cos(ang) * sd);
                if (2 * q + 1 < size) dst[2 * q + 1] = (float)(rad * std::sin(ang) * sd);
            }
        };
        unsigned nt = std::thread::hardware_concurrency();
        if (nt == 0) nt = 1;
        if (nt > 16) nt = 16;
        if (pairs < (1 << 16) || nt == 1) {
            fill(0, pairs);
        } else {
            std::vector<std::thread> pool;
            const int64_t per = (pairs + nt - 1) / nt;
            for (unsigned i = 0; i < nt; ++i) {
                const int64_t a = (int64_t)i * per, b = a + per < pairs ? a + per : pairs;
                if (a < b) pool.emplace_back(fill, a, b);
            }
            for (auto& th : pool) th.join();
        }
    }
}

// ---------------------------------------------------------------- graph
static int out_extent(int in, int k, int stride, int pad) { return (in + 2 * pad - k) / stride + 1; }

int Graph::add_tensor(int H, int W, int C) {
    Tensor t;
    t.H = H; t.W = W; t.C = C;
    tensors.push_back(t);
    return (int)tensors.size() - 1;
}

int Graph::conv(int x, int K, int R, int stride, int pad, bool bias, bool relu, const std::string& name) {
    const Tensor tx = tensors[(size_t)x];
    Op op;
    op.kind = OP_CONV; op.x = x; op.K = K; op.R = R; op.S = R; op.stride = stride; op.pad = pad;
    op.bias = bias; op.relu = relu; op.name = name;
    op.w_off = P;
    const int64_t wsize = (int64_t)K * R * R * tx.C;
    params.push_back({name + ".w", P, wsize, (int64_t)tx.C * R * R, false});
    P += wsize;
    if (bias) {
        op.b_off = P;
        params.push_back({name + ".b", P, K, 0, false});
        P += K;
    }
    op.y = add_tensor(out_extent(tx.H, R, stride, pad), out_extent(tx.W, R, stride, pad), K);
    ops.push_back(op);
    return op.y;
}

int Graph::bn(int x, bool relu, int res, const std::string& name) {
    const Tensor tx = tensors[(size_t)x];
    Op op;
    op.kind = OP_BN; op.x = x; op.res = res; op.relu = relu; op.K = tx.C; op.name = name;
    op.w_off = P; op.b_off = P + tx.C; op.run_off = R;
    params.push_back({name + ".g", P, tx.C, 0, true});
    params.push_back({name + ".b", P + tx.C, tx.C, 0, false});
    P += 2 * tx.C;
    R += 2 * tx.C;
    op.y = add_tensor(tx.H, tx.W, tx.C);
    ops.push_back(op);
    return op.y;
}

int Graph::maxpool(int x, int k, int stride, int pad) {
    const Tensor tx = tensors[(size_t)x];
    Op op;
    op.kind = OP_MAXPOOL; op.x = x; op.R = k; op.S = k; op.stride = stride; op.pad = pad;
    op.y = add_tensor(out_extent(tx.H, k, stride, pad), out_extent(tx.W, k, stride, pad), tx.C);
    ops.push_back(op);
    return op.y;
}

int Graph::gavgpool(int x) {
    const Tensor tx = tensors[(size_t)x];
    Op op;
    op.kind = OP_GAVGPOOL; op.x = x;
    op.y = add_tensor(1, 1, tx.C);
    ops.push_back(op);
    return op.y;
}

int Graph::flatten(int x) {
    const Tensor tx = tensors[(size_t)x];
    const int y = add_tensor(1, 1, tx.H * tx.W * tx.C);
    tensors[(size_t)y].alias_of = tensors[(size_t)x].alias_of >= 0 ? tensors[(size_t)x].alias_of : x;
    return y;
}

void Graph::loss(int x) {
    Op op;
    op.kind = OP_LOSS; op.x = x;
    ops.push_back(op);
    logits = x;
    tensors[(size_t)x].fp32 = true;
    classes = tensors[(size_t)x].C;
}

// 2 flops per multiply-add, forward + input-gradient + weight-gradient
// contractions; the first layer has no input gradient.
double Graph::flops_per_sample() const {
    double f = 0;
    for (const Op& op : ops) {
        if (op.kind != OP_CONV) continue;
        const Tensor& ty = tensors[(size_t)op.y];
        const Tensor& tx = tensors[(size_t)op.x];
        const double macs = (double)ty.H * ty.W * op.K * op.R * op.S * tx.C;
        const bool first = (op.x == 0) || (tensors[(size_t)op.x].alias_of == 0);
        f += 2.0 * macs * (first ? 2.0 : 3.0);
    }
    return f;
}

static int pick(int v, int dflt) { return v > 0 ? v : dflt; }

static void build_mlp(const edl_config& c, Graph& g) {
    const int H = pick(c.H, 1), W = pick(c.W, 1), C = pick(c.C, 784);
    const int h1 = pick(c.arch[0], 256), h2 = pick(c.arch[1], 256), classes = pick(c.classes, 10);
    int t = g.flatten(g.add_tensor(H, W, C));
    t = g.conv(t, h1, 1, 1, 0, true, true, "fc1");
    t = g.conv(t, h2, 1, 1, 0, true, true, "fc2");
    t = g.conv(t, classes, 1, 1, 0, true, false, "fc3");
    g.loss(t);
}

static std::string blk(int stage, int block) {
    char buf[32];
    snprintf(buf, sizeof(buf), "s%d.b%d", stage, block);
    return buf;
}

// CIFAR-style residual net: 3x3 stem, `stages` stages of `blocks` basic blocks,
// width doubling and stride 2 at each stage change, where the shortcut is a
// strided 1x1 projection with its own batch norm.
static void build_resnet20(const edl_config& c, Graph& g) {
    const int H = pick(c.H, 32), W = pick(c.W, 32), C = pick(c.C, 3), classes = pick(c.classes, 10);
    const int w0 = pick(c.arch[0], 16), stages = pick(c.arch[1], 3), blocks = pick(c.arch[2], 3);
    int t = g.conv(g.add_tensor(H, W, C), w0, 3, 1, 1, false, false, "stem.conv");
    t = g.bn(t, true, -1, "stem.bn");
    int cin = w0;
    for (int s = 0; s < stages; ++s) {
        const int width = w0 << s;
        for (int b = 0; b < blocks; ++b) {
            const int stride = (s > 0 && b == 0) ? 2 : 1;
            const std::string nm = blk(s + 1, b + 1);
            int u = g.conv(t, width, 3, stride, 1, false, false, nm + ".conv1");
            u = g.bn(u, true, -1, nm + ".bn1");
            u = g.conv(u, width, 3, 1, 1, false, false, nm + ".conv2");
            int sc = t;
            if (stride != 1 || cin != width) {
                sc = g.conv(t, width, 1, stride, 0, false, false, nm + ".proj");
                sc = g.bn(sc, false, -1, nm + ".projbn");
            }
            t = g.bn(u, true, sc, nm + ".bn2");
            cin = width;
        }
    }
    t = g.gavgpool(t);
    t = g.conv(t, classes, 1, 1, 0, true, false, "fc");
    g.loss(t);
}

// Bottleneck residual net: 7x7/2 stem, 3x3/2 max pool, stages of
// 1x1 - 3x3 - 1x1 blocks (the 3x3 carries the stride), projection shortcut on
// the first block of every stage.
static void build_resnet50(const edl_config& c, Graph& g) {
    const int H = pick(c.H, 224), W = pick(c.W, 224), C = pick(c.C, 3), classes = pick(c.classes, 1000);
    const int base = pick(c.arch[0], 64);
    int nb[4] = {3, 4, 6, 3};
    if (c.arch[1] > 0) for (int i = 0; i < 4; ++i) nb[i] = c.arch[1 + i];
    int t = g.conv(g.add_tensor(H, W, C), base, 7, 2, 3, false, false, "stem.conv");
    t = g.bn(t, true, -1, "stem.bn");
    t = g.maxpool(t, 3, 2, 1);
    for (int s = 0; s < 4 && nb[s] > 0; ++s) {
        const int width = base << s;
        for (int b = 0; b < nb[s]; ++b) {
            const int stride = (s > 0 && b == 0) ? 2 : 1;
            const std::string nm = blk(s + 1, b + 1);
            int u = g.conv(t, width, 1, 1, 0, false, false, nm + ".conv1");
            u = g.bn(u, true, -1, nm + ".bn1");
            u = g.conv(u, width, 3, stride, 1, false, false, nm + ".conv2");
            u = g.bn(u, true, -1, nm + ".bn2");
            u = g.conv(u, 4 * width, 1, 1, 0, false, false, nm + ".conv3");
            int sc = t;
            if (b == 0) {
                sc = g.conv(t, 4 * width, 1, stride, 0, false, false, nm + ".proj");
                sc = g.bn(sc, false, -1, nm + ".projbn");
            }
            t = g.bn(u, true, sc, nm + ".bn3");
        }
    }
    t = g.gavgpool(t);
    t = g.conv(t, classes, 1, 1, 0, true, false, "fc");
    g.loss(t);
}

// Biased 3x3 convolutions with ReLU in five groups (2,2,3,3,3 of them for the
// 16-layer net, 2,2,4,4,4 for the 19-layer one), a 2x2/2 max pool after each
// group, three fully connected layers.  No batch norm, no dropout.
static void build_vgg16(const edl_config& c, Graph& g) {
    const int H = pick(c.H, 224), W = pick(c.W, 224), C = pick(c.C, 3), classes = pick(c.classes, 1000);
    const int base = pick(c.arch[0], 64), fc = pick(c.arch[1], 4096);
    int reps[5] = {2, 2, 3, 3, 3};
    if (c.arch[2] > 0) for (int i = 0; i < 5; ++i) reps[i] = c.arch[2 + i];
    const int mult[5] = {1, 2, 4, 8, 8};
    int t = g.add_tensor(H, W, C);
    int i = 0;
    char nm[16];
    for (int grp = 0; grp < 5; ++grp) {
        for (int r = 0; r < reps[grp]; ++r) {
            snprintf(nm, sizeof(nm), "conv%d", ++i);
            t = g.conv(t, base * mult[grp], 3, 1, 1, true, true, nm);
        }
        t = g.maxpool(t, 2, 2, 0);
    }
    t = g.flatten(t);
    t = g.conv(t, fc, 1, 1, 0, true, true, "fc1");
    t = g.conv(t, fc, 1, 1, 0, true, true, "fc2");
    t = g.conv(t, classes, 1, 1, 0, true, false, "fc3");
    g.loss(t);
}

// Five biased convolutions with ReLU (11x11/4 pad 2, 5x5 pad 2, three 3x3
// pad 1; base x {1,3,6,4,4} channels), a 3x3/2 max pool after the first, the
// second and the fifth, three fully connected layers.  The single-tower form
// without response normalisation; no dropout.
static void build_alexnet(const edl_config& c, Graph& g) {
    const int H = pick(c.H, 224), W = pick(c.W, 224), C = pick(c.C, 3), classes = pick(c.classes, 1000);
    const int base = pick(c.arch[0], 64), fc = pick(c.arch[1], 4096);
    int t = g.add_tensor(H, W, C);
    t = g.conv(t, base, 11, 4, 2, true, true, "conv1");
    t = g.maxpool(t, 3, 2, 0);
    t = g.conv(t, 3 * base, 5, 1, 2, true, true, "conv2");
    t = g.maxpool(t, 3, 2, 0);
    t = g.conv(t, 6 * base, 3, 1, 1, true, true, "conv3");
    t = g.conv(t, 4 * base, 3, 1, 1, true, true, "conv4");
    t = g.conv(t, 4 * base, 3, 1, 1, true, true, "conv5");
    t = g.maxpool(t, 3, 2, 0);
    t = g.flatten(t);
    t = g.conv(t, fc, 1, 1, 0, true, true, "fc1");
    t = g.conv(t, fc, 1, 1, 0, true, true, "fc2");
    t = g.conv(t, classes, 1, 1, 0, true, false, "fc3");
    g.loss(t);
}

int build_graph(const edl_config& cfg, Graph& g) {
    g = Graph();
    switch (cfg.model) {
        case EDL_MODEL_MLP: build_mlp(cfg, g); break;
        case EDL_MODEL_RESNET20: build_resnet20(cfg, g); break;
        case EDL_MODEL_RESNET50: build_resnet50(cfg, g); break;
        case EDL_MODEL_VGG16: build_vgg16(cfg, g); break;
        case EDL_MODEL_ALEXNET: build_alexnet(cfg, g); break;
        default: set_error("unknown model %d", cfg.model); return EDL_EINVAL;
    }
    for (const Tensor& t : g.tensors)
        if (t.H <= 0 || t.W <= 0 || t.C <= 0) {
            set_error("input image too small for this model");
            return EDL_EINVAL;
        }
    return EDL_OK;
}

}  // namespace edl
