// C boundary and step executor: carves the caller's arena, runs the layer
// list forward and backward for each worker's shard, then the fused
// aggregation + update.  See include/edl.h for the contract of every call.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <vector>

#include "graph.h"
#include "kernels.h"
#include "profiler.h"
#include "tune.h"

using namespace edl;

#define HIP_TRY(expr)                                                                      \
    do {                                                                                   \
        hipError_t e_ = (expr);                                                            \
        if (e_ != hipSuccess) {                                                            \
            set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, __LINE__); \
            return EDL_EHIP;                                                               \
        }                                                                                  \
    } while (0)

// Scratch for edl_step_static_scratch (callers that cannot bring or allocate a scratch piece): one fixed buffer
// per GPU, held from the time the library's code is loaded on that GPU until the process ends.  In host code
// this name is only a handle for hipGetSymbolAddress; the device address is taken once per device in edl_init
// and kept in g_static_scratch, and that pointer is what kernels and copies are given.
static __device__ __align__(256) unsigned char scratch[EDL_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
void* g_static_scratch[kMaxDevices] = {};     // per device: address of that device's copy of `scratch`

constexpr int64_t kAlign = 256;
constexpr int kIdxSlots = 4;
constexpr int kReadyEvents = 64;   // ring of "dy is final" events for the second stream
constexpr int kChunkEvents = 64;   // ring of "these weight gradients are final" events for the update stream
constexpr int kBranchEvents = 16;  // ring of event pairs around a shortcut branch on the second side stream

int64_t align_up(int64_t v, int64_t a = kAlign) { return (v + a - 1) / a * a; }

// header of the state image (little endian, packed by construction)
struct SnapshotHeader {
    uint32_t magic, version, model, dtype;
    uint64_t seed;
    int64_t N, B, step, epoch, step_in_epoch;
    float lr, momentum, wd;
    uint32_t optimizer;
    int64_t P, R;
    float beta2, eps;      // Adam only, else 0
};
static_assert(sizeof(SnapshotHeader) == 104, "snapshot header layout");

struct Layout {
    int64_t params = 0, momentum = 0, second = -1, running = 0, shadow = 0, grads = 0, grad_stride = 0;
    int64_t idx = 0, labels = 0, row_loss = 0, losses = 0, partial = 0, partial_held = 0, coef = 0, wgrad_scratch = 0;
    int64_t partial_side = 0, coef_side = 0, wide_sums_side = 0, splitk_side = 0;   // the branch stream's own scratch
    int64_t wide_sums = 0, wide_sums_floats = 0;   // partial column sums of launches with more row tiles than `partial` holds
    int64_t wgrad_scratch_bytes = 0;
    int64_t wgrad_scratch2 = 0;          // for the few weight gradients that run on the main stream beside the second one
    // partial sums of forward / dgrad reductions that are cut; apart from the weight-gradient
    // scratch because weight gradients may run on the second stream meanwhile
    int64_t splitk_scratch = 0, splitk_scratch_bytes = 0;
    int64_t ttable = 0;                  // TransposeEntry[] for the one-launch weight transpose
    int64_t scratch_lo = 0, scratch_hi = 0;   // the kernels' scratch pieces lie in [scratch_lo, scratch_hi)
    int cpad = 0;                        // channels of the stored input images (>= the logical count, see input_pad)
    std::vector<int64_t> wpad;           // per op: zero-padded weight copy of a convolution on padded images (-1 if none)
    int64_t dwpad = 0;                   // float32 gradient of such weights before it is compacted
    std::vector<int64_t> act, grad;      // per tensor (storage owners only; -1 otherwise)
    std::vector<int64_t> wT;             // per op: transposed weight copy (-1 if not needed)
    std::vector<int64_t> bn_save;        // per op
    std::vector<int64_t> pool_arg;       // per op
    int64_t total = 0;
};

int validate(const edl_config& c) {
    if (c.dtype != EDL_DTYPE_F32 && c.dtype != EDL_DTYPE_BF16) { set_error("unknown dtype %d", c.dtype); return EDL_EINVAL; }
    if (c.N <= 0 || c.B <= 0 || c.p_max <= 0 || c.max_shard <= 0) { set_error("N, B, p_max, max_shard must be positive"); return EDL_EINVAL; }
    if (c.p_max > kMaxP) { set_error("p_max %d exceeds %d", c.p_max, kMaxP); return EDL_EINVAL; }
    if (c.N % c.B) { set_error("N=%lld is not a multiple of B=%lld", (long long)c.N, (long long)c.B); return EDL_EINDIVISIBLE; }
    if (c.max_shard > c.B) { set_error("max_shard exceeds B"); return EDL_EINVAL; }
    if (c.optimizer != EDL_OPT_MOMENTUM && c.optimizer != EDL_OPT_ADAM) { set_error("unknown optimizer %d", c.optimizer); return EDL_EINVAL; }
    if (c.optimizer == EDL_OPT_ADAM &&
        !(c.momentum >= 0.f && c.momentum < 1.f && c.beta2 >= 0.f && c.beta2 < 1.f && c.eps >= 0.f)) {
        set_error("Adam needs 0 <= beta1 (momentum), beta2 < 1 and eps >= 0");
        return EDL_EINVAL;
    }
    return EDL_OK;
}

int storage_of(const Graph& g, int t) { return g.tensors[(size_t)t].alias_of >= 0 ? g.tensors[(size_t)t].alias_of : t; }

ConvGeom geom_of(const Graph& g, const Op& op, int n) {
    const Tensor& tx = g.tensors[(size_t)op.x];
    const Tensor& ty = g.tensors[(size_t)op.y];
    ConvGeom q;
    q.N = n; q.H = tx.H; q.W = tx.W; q.C = tx.C;
    q.K = op.K; q.R = op.R; q.S = op.S; q.stride = op.stride; q.pad = op.pad; q.Ho = ty.H; q.Wo = ty.W;
    return q;
}

// Images whose channel count is not a multiple of the 16-byte vector (RGB) are
// stored with every pixel padded to one vector, so that the first convolution
// runs on the vector path.  Not when a flattened view of the images exists.
int input_pad(const edl_config& c, const Graph& g) {
    const int vec = c.dtype == EDL_DTYPE_BF16 ? 8 : 4;
    const int C = g.tensors[0].C;
    if (C % vec == 0 || C > vec) return C;
    for (const Tensor& t : g.tensors)
        if (t.alias_of == 0) return C;
    return vec;
}

ConvGeom geom_padded(const Graph& g, const Op& op, int n, int cpad) {
    ConvGeom q = geom_of(g, op, n);
    if (op.x == 0) q.C = cpad;
    return q;
}

void plan_layout(const edl_config& c, const Graph& g, Layout& L) {
    const int64_t esz = c.dtype == EDL_DTYPE_BF16 ? 2 : 4;
    L.cpad = input_pad(c, g);
    int64_t o = 0;
    auto take = [&](int64_t bytes) { const int64_t at = o; o += align_up(bytes); return at; };
    // The arrays the update kernel walks side by side (w, v, the bf16 copy, the p gradient buffers) start on 4 KB
    // boundaries, alternately even and odd ones (offset bit 12): a workgroup touches the same offset of every
    // array at the same time, and arrays that all start 8 KB-aligned meet in the same half of the memory system
    // (measured: 5.6 -> 6.2 TB/s for the update; the arena itself should start on an 8 KB boundary for this to
    // hold, as torch's large allocations do).
    auto take_page = [&](int64_t bytes, int odd) {
        o = (o + 8191) / 8192 * 8192 + (odd ? 4096 : 0);
        const int64_t at = o;
        o += align_up(bytes);
        return at;
    };
    L.params = take_page(4 * g.P, 0);
    L.momentum = take_page(4 * g.P, 1);
    if (c.optimizer == EDL_OPT_ADAM) L.second = take_page(4 * g.P, 0);
    L.shadow = c.dtype == EDL_DTYPE_BF16 ? take_page(2 * g.P, c.optimizer == EDL_OPT_ADAM ? 1 : 0) : -1;
    // consecutive gradient buffers an odd number of 4 KB pages apart, the first one on an odd page
    L.grad_stride = ((4 * g.P + 8191) / 8192 * 8192 + 4096) / 4;
    L.grads = take_page(4 * L.grad_stride * c.p_max, 1);
    L.running = take(4 * std::max<int64_t>(g.R, 1));
    L.idx = take(8 * c.B);
    L.labels = take(4 * (int64_t)c.max_shard);
    L.losses = take(4 * kMaxP);
    int cmax = 1;
    for (const Op& op : g.ops)
        if (op.kind == OP_CONV || op.kind == OP_BN) cmax = std::max(cmax, op.K);
    const size_t nt = g.tensors.size();
    L.act.assign(nt, -1);
    L.grad.assign(nt, -1);
    for (size_t t = 0; t < nt; ++t) {
        if (g.tensors[t].alias_of >= 0) continue;
        int64_t elems = g.tensors[t].elems() * c.max_shard;
        if (t == 0) elems = (int64_t)g.tensors[0].H * g.tensors[0].W * L.cpad * c.max_shard;
        L.act[t] = take(elems * (g.tensors[t].fp32 ? 4 : esz));
        if (t != 0) L.grad[t] = take(elems * esz);
    }
    const size_t no = g.ops.size();
    L.wT.assign(no, -1);
    L.wpad.assign(no, -1);
    int64_t dwpad_bytes = 16;
    L.bn_save.assign(no, -1);
    L.pool_arg.assign(no, -1);
    L.wgrad_scratch_bytes = 0;
    L.splitk_scratch_bytes = 0;
    for (size_t i = 0; i < no; ++i) {
        const Op& op = g.ops[i];
        if (op.kind == OP_CONV) {
            const Tensor& tx = g.tensors[(size_t)op.x];
            if (storage_of(g, op.x) != 0) L.wT[i] = take((int64_t)op.K * op.R * op.S * tx.C * esz);
            else if (op.x == 0 && L.cpad != tx.C) {
                L.wpad[i] = take((int64_t)op.K * op.R * op.S * L.cpad * esz);
                dwpad_bytes = std::max<int64_t>(dwpad_bytes, (int64_t)op.K * op.R * op.S * L.cpad * 4);
            }
            L.wgrad_scratch_bytes = std::max<int64_t>(L.wgrad_scratch_bytes,
                                                      (int64_t)conv_wgrad_scratch_bytes(geom_padded(g, op, c.max_shard, L.cpad)));
            // the cut of a forward / dgrad reduction depends on the shard size: cover every size up to the largest
            for (int n = 1; n <= c.max_shard; n = n < 8 ? n + 1 : n + n / 4)
                L.splitk_scratch_bytes = std::max<int64_t>(L.splitk_scratch_bytes,
                                                           (int64_t)conv_splitk_scratch_bytes(c.dtype, geom_of(g, op, n)));
            L.splitk_scratch_bytes = std::max<int64_t>(L.splitk_scratch_bytes,
                                                       (int64_t)conv_splitk_scratch_bytes(c.dtype, geom_of(g, op, c.max_shard)));
            L.wide_sums_floats = std::max<int64_t>(L.wide_sums_floats,
                                                   (int64_t)conv_wide_sums_floats(c.dtype, geom_padded(g, op, c.max_shard, L.cpad)));
        } else if (op.kind == OP_BN) {
            L.bn_save[i] = take(4 * 2 * (int64_t)op.K);
        } else if (op.kind == OP_MAXPOOL) {
            L.pool_arg[i] = take(g.tensors[(size_t)op.y].elems() * c.max_shard);
        }
    }
    // The kernels' scratch (partial results that live inside one pass), in one contiguous piece
    // [scratch_lo, scratch_hi): a caller without an arena piece for it can run the same pass on the library's
    // static buffer (edl_step_static_scratch).
    L.scratch_lo = o;
    L.row_loss = take(4 * (int64_t)c.max_shard);
    L.partial = take(4 * 2 * (int64_t)kRedRowBlocks * cmax);
    // a second one for sums that wait while another batch norm runs (a block's last convolution, whose
    // batch norm comes after the projection shortcut's)
    L.partial_held = take(4 * 2 * (int64_t)kRedRowBlocks * cmax);
    L.coef = take(4 * 2 * (int64_t)cmax);
    // the same pair for the projection shortcut's batch norm while it runs on the branch stream beside the main one
    L.partial_side = take(4 * 2 * (int64_t)kRedRowBlocks * cmax);
    L.coef_side = take(4 * 2 * (int64_t)cmax);
    L.wgrad_scratch = take(std::max<int64_t>(L.wgrad_scratch_bytes, 16));
    L.wgrad_scratch2 = take(std::max<int64_t>(L.wgrad_scratch_bytes, 16));
    L.wide_sums = take(std::max<int64_t>(4 * L.wide_sums_floats, 16));
    L.splitk_scratch = take(std::max<int64_t>(L.splitk_scratch_bytes, 16));
    // the branch stream cuts reductions and keeps wide sums exactly as the main stream would (same results, bit
    // for bit, whichever stream a layer runs on), in buffers of its own
    L.wide_sums_side = take(std::max<int64_t>(4 * L.wide_sums_floats, 16));
    L.splitk_side = take(std::max<int64_t>(L.splitk_scratch_bytes, 16));
    L.dwpad = take(dwpad_bytes);
    L.scratch_hi = o;
    L.ttable = take((int64_t)sizeof(TransposeEntry) * 2 * std::max<size_t>(no, 1));   // element-wise entries, then vector ones
    L.total = o;
}

}  // namespace

struct edl_handle {
    edl_config cfg;
    uint64_t seed;
    Graph g;
    Layout L;
    char* arena;
    hipStream_t st;
    const float* data_x = nullptr;
    const int32_t* data_y = nullptr;
    edl_progress prog = {0, 0, 0};
    bool weights_dirty = true;
    // cached permutation of the current epoch
    int64_t perm_epoch = -1;
    std::vector<int64_t> perm;
    int t_entries = 0, t_tiles = 0;      // one-launch weight transpose (element-wise entries)
    double t_bytes = 0;
    int tv_entries = 0, tv_tiles = 0;    // ... and the bf16 layers of vector-friendly shape
    double tv_bytes = 0;
    // pinned staging
    int64_t* idx_host[kIdxSlots] = {nullptr, nullptr, nullptr, nullptr};
    hipEvent_t idx_event[kIdxSlots] = {};
    int idx_slot = 0;
    float* loss_host = nullptr;
    std::vector<int> readers;            // per tensor storage: how many layers read it (as input or as residual)
    std::vector<int> first_reader;       // per tensor storage: the first of them in the layer list (the last to run backward)
    // shard sizes of the last edl_gradients (what edl_apply weighs the gradient buffers by)
    std::vector<int64_t> shard_n;
    bool shards_equal = true;
    bool grads_pending = false;          // edl_gradients has run and edl_apply has not consumed its buffers yet
    // second stream for the weight gradients (null: everything on st); own_streams: created here, not the caller's
    hipStream_t side = nullptr;
    bool own_streams = false;
    hipEvent_t ev_ready[kReadyEvents] = {};
    hipEvent_t ev_side_done = nullptr;
    int ev_slot = 0;
    // The update of the parameters whose gradients are final starts during the last backward pass of a step,
    // on a stream of its own: `early_p` > 0 asks the backward pass for it (the p of the step), `applied_from`
    // is the first parameter already updated (P = none yet).
    hipStream_t upd = nullptr;
    hipEvent_t ev_chunk[kChunkEvents] = {};
    hipEvent_t ev_upd_done = nullptr;
    int chunk_slot = 0;
    int early_p = 0;
    int64_t applied_from = 0;

    // where the kernels' scratch lives during the current call: the arena piece (null), or another buffer of
    // the same layout
    char* scratch_base = nullptr;
    int device = -1;
    std::vector<char> written;           // backward pass: which gradient buffers hold something (per tensor)
    std::vector<char> op_done;           // a pass: layers already launched out of list order (on the branch stream)
    // backward pass, per tensor: where the gradient "already there" is to be read from if not from the tensor's
    // own gradient buffer (an identity shortcut's part is the masked gradient of the block's output itself)
    std::vector<const void*> grad_alias;
    // The projection shortcut of a residual block (a convolution and its batch norm) depends only on the block's
    // input (forward) / on the gradient the block's last batch norm leaves for it (backward), so it runs on the
    // second side stream beside the main branch: ev_branch_go releases it, ev_branch_done joins it.
    hipEvent_t ev_branch_go[kBranchEvents] = {}, ev_branch_done[kBranchEvents] = {};
    int branch_slot = 0;
    hipEvent_t ev_tr_go = nullptr, ev_tr_done = nullptr;   // around the weight transposes on the weight-gradient stream
    bool transposes_pending = false;

    template <typename T> T* at(int64_t off) const { return reinterpret_cast<T*>(arena + off); }
    // a piece of the kernels' scratch (off is its arena offset)
    template <typename T> T* sc(int64_t off) const {
        return reinterpret_cast<T*>(scratch_base ? scratch_base + (off - L.scratch_lo) : arena + off);
    }
    float* w() const { return at<float>(L.params); }
    float* v() const { return at<float>(L.momentum); }
    float* s2() const { return at<float>(L.second); }                     // Adam only
    bool adam() const { return cfg.optimizer == EDL_OPT_ADAM; }
    int64_t state_floats() const { return (adam() ? 3 : 2) * g.P + g.R; }   // w, optimizer slots, running
    float* running() const { return at<float>(L.running); }
    float* grad_buf(int k) const { return at<float>(L.grads) + (int64_t)k * L.grad_stride; }
    void* act(int t) const { return arena + L.act[(size_t)storage_of(g, t)]; }
    void* grad(int t) const { return arena + L.grad[(size_t)storage_of(g, t)]; }
};

extern "C" {

const char* edl_last_error(void) { return get_error(); }

int32_t edl_query(const edl_config* cfg, edl_sizes* out) {
    if (!cfg || !out) { set_error("null argument"); return EDL_EINVAL; }
    int rc = validate(*cfg);
    if (rc) return rc;
    Graph g;
    rc = build_graph(*cfg, g);
    if (rc) return rc;
    Layout L;
    plan_layout(*cfg, g, L);
    out->P = g.P;
    out->R = g.R;
    out->params_off = L.params;
    out->momentum_off = L.momentum;
    out->running_off = L.running;
    out->grads_off = L.grads;
    out->grad_stride = L.grad_stride;
    out->arena_bytes = L.total;
    out->snapshot_bytes = EDL_SNAPSHOT_HEADER_BYTES + 4 * ((cfg->optimizer == EDL_OPT_ADAM ? 3 : 2) * g.P + g.R);
    out->flops_per_sample = g.flops_per_sample();
    out->second_off = L.second;
    out->shadow_off = L.shadow;
    out->scratch_bytes = L.scratch_hi - L.scratch_lo;
    return EDL_OK;
}

int32_t edl_tensor_count(const edl_config* cfg, int32_t* out_count) {
    if (!cfg || !out_count) { set_error("null argument"); return EDL_EINVAL; }
    Graph g;
    const int rc = build_graph(*cfg, g);
    if (rc) return rc;
    *out_count = (int32_t)g.params.size();
    return EDL_OK;
}

int32_t edl_tensor_info(const edl_config* cfg, int32_t i, char* name_buf, size_t name_cap, int64_t* out_offset,
                        int64_t* out_size, int64_t* out_fan_in) {
    if (!cfg) { set_error("null argument"); return EDL_EINVAL; }
    Graph g;
    const int rc = build_graph(*cfg, g);
    if (rc) return rc;
    if (i < 0 || (size_t)i >= g.params.size()) { set_error("tensor index %d out of range", i); return EDL_ERANGE; }
    const ParamTensor& pt = g.params[(size_t)i];
    if (name_buf && name_cap) snprintf(name_buf, name_cap, "%s", pt.name.c_str());
    if (out_offset) *out_offset = pt.off;
    if (out_size) *out_size = pt.size;
    if (out_fan_in) *out_fan_in = pt.fan_in;
    return EDL_OK;
}

int32_t edl_init_params_host(const edl_config* cfg, uint64_t seed, float* out_params) {
    if (!cfg || !out_params) { set_error("null argument"); return EDL_EINVAL; }
    Graph g;
    const int rc = build_graph(*cfg, g);
    if (rc) return rc;
    he_init(g, seed, out_params);
    return EDL_OK;
}

int32_t edl_shard_host(uint64_t seed, int64_t N, int64_t B, int32_t p, int64_t epoch, int64_t step_in_epoch,
                       int64_t* out_idx, int64_t* out_off) {
    if (!out_idx || !out_off) { set_error("null argument"); return EDL_EINVAL; }
    if (N <= 0 || B <= 0 || p <= 0 || epoch < 0) { set_error("N, B, p must be positive and epoch non-negative"); return EDL_EINVAL; }
    if (B % p || N % B) { set_error("B=%lld must divide by p=%d and N=%lld by B", (long long)B, p, (long long)N); return EDL_EINDIVISIBLE; }
    if (step_in_epoch < 0 || step_in_epoch >= N / B) { set_error("step_in_epoch %lld outside the epoch", (long long)step_in_epoch); return EDL_ERANGE; }
    std::vector<int64_t> perm;
    epoch_permutation(seed, epoch, N, perm);
    memcpy(out_idx, perm.data() + step_in_epoch * B, sizeof(int64_t) * (size_t)B);
    for (int k = 0; k <= p; ++k) out_off[k] = (int64_t)k * (B / p);
    return EDL_OK;
}

static int refresh_weight_copies(edl_handle* h) {
    // the bf16 copy is written by the update kernel; after init / restore /
    // set_params it is made here.  The transposed copies always are.
    const int dt = h->cfg.dtype;
    if (dt == EDL_DTYPE_BF16) launch_cast_bf16(h->w(), h->at<uint16_t>(h->L.shadow), h->g.P, h->st);
    return EDL_OK;
}

// The transposed weight copies (read by the input-gradient passes only) on stream tst; the zero-padded copy of
// the first convolution's weights (read by the forward pass) on the job's stream.
static void transpose_weights(edl_handle* h, hipStream_t tst) {
    launch_weight_transpose_all(h->cfg.dtype, h->w(), h->arena, h->at<TransposeEntry>(h->L.ttable), h->t_entries,
                                h->t_tiles, h->t_bytes, tst);
    if (h->tv_entries > 0)
        launch_weight_transpose_bf16(h->at<uint16_t>(h->L.shadow), h->arena, h->at<TransposeEntry>(h->L.ttable) + h->g.ops.size(),
                                     h->tv_entries, h->tv_tiles, h->tv_bytes, tst);
    for (size_t i = 0; i < h->g.ops.size(); ++i)
        if (h->L.wpad[i] >= 0) {
            const Op& op = h->g.ops[i];
            launch_pad_weights(h->cfg.dtype, h->w() + op.w_off, h->arena + h->L.wpad[i], (int64_t)op.K * op.R * op.S,
                               h->g.tensors[0].C, h->L.cpad, h->st);
        }
}

static int init_device_state(edl_handle* h);

// events that order the side streams against the job's stream (created once, whoever owns the streams)
static int create_side_events(edl_handle* h) {
    for (int e = 0; e < kReadyEvents; ++e)
        if (!h->ev_ready[e]) HIP_TRY(hipEventCreateWithFlags(&h->ev_ready[e], hipEventDisableTiming));
    if (!h->ev_side_done) HIP_TRY(hipEventCreateWithFlags(&h->ev_side_done, hipEventDisableTiming));
    for (int e = 0; e < kChunkEvents; ++e)
        if (!h->ev_chunk[e]) HIP_TRY(hipEventCreateWithFlags(&h->ev_chunk[e], hipEventDisableTiming));
    if (!h->ev_upd_done) HIP_TRY(hipEventCreateWithFlags(&h->ev_upd_done, hipEventDisableTiming));
    if (!h->ev_tr_go) HIP_TRY(hipEventCreateWithFlags(&h->ev_tr_go, hipEventDisableTiming));
    if (!h->ev_tr_done) HIP_TRY(hipEventCreateWithFlags(&h->ev_tr_done, hipEventDisableTiming));
    for (int e = 0; e < kBranchEvents; ++e) {
        if (!h->ev_branch_go[e]) HIP_TRY(hipEventCreateWithFlags(&h->ev_branch_go[e], hipEventDisableTiming));
        if (!h->ev_branch_done[e]) HIP_TRY(hipEventCreateWithFlags(&h->ev_branch_done[e], hipEventDisableTiming));
    }
    return EDL_OK;
}

// waits for the side streams and lets go of them (destroys them only if the library made them)
static void release_side_streams(edl_handle* h) {
    if (h->side) (void)hipStreamSynchronize(h->side);
    if (h->upd) (void)hipStreamSynchronize(h->upd);
    if (h->own_streams) {
        if (h->side) (void)hipStreamDestroy(h->side);
        if (h->upd) (void)hipStreamDestroy(h->upd);
    }
    h->side = nullptr;
    h->upd = nullptr;
    h->own_streams = false;
}

// frees whatever of the handle's resources exist (also a half-built handle) and the handle
static void destroy_handle(edl_handle* h) {
    (void)hipStreamSynchronize(h->st);
    release_side_streams(h);
    for (int s = 0; s < kIdxSlots; ++s) {
        if (h->idx_host[s]) (void)hipHostFree(h->idx_host[s]);
        if (h->idx_event[s]) (void)hipEventDestroy(h->idx_event[s]);
    }
    if (h->loss_host) (void)hipHostFree(h->loss_host);
    for (int e = 0; e < kReadyEvents; ++e)
        if (h->ev_ready[e]) (void)hipEventDestroy(h->ev_ready[e]);
    for (int e = 0; e < kChunkEvents; ++e)
        if (h->ev_chunk[e]) (void)hipEventDestroy(h->ev_chunk[e]);
    if (h->ev_side_done) (void)hipEventDestroy(h->ev_side_done);
    if (h->ev_upd_done) (void)hipEventDestroy(h->ev_upd_done);
    if (h->ev_tr_go) (void)hipEventDestroy(h->ev_tr_go);
    if (h->ev_tr_done) (void)hipEventDestroy(h->ev_tr_done);
    for (int e = 0; e < kBranchEvents; ++e) {
        if (h->ev_branch_go[e]) (void)hipEventDestroy(h->ev_branch_go[e]);
        if (h->ev_branch_done[e]) (void)hipEventDestroy(h->ev_branch_done[e]);
    }
    delete h;
}

int32_t edl_init(edl_handle** out, const edl_config* cfg, uint64_t seed, void* dev_arena, size_t arena_bytes,
                 void* hip_stream) {
    if (!out || !cfg || !dev_arena) { set_error("null argument"); return EDL_EINVAL; }
    int rc = validate(*cfg);
    if (rc) return rc;
    if (((uintptr_t)dev_arena) % kAlign) { set_error("arena must be 256-byte aligned"); return EDL_EINVAL; }
    edl_handle* h = new edl_handle();
    h->cfg = *cfg;
    h->seed = seed;
    rc = build_graph(*cfg, h->g);
    if (rc) { delete h; return rc; }
    plan_layout(*cfg, h->g, h->L);
    if ((int64_t)arena_bytes < h->L.total) {
        set_error("arena of %zu bytes is smaller than the %lld needed", arena_bytes, (long long)h->L.total);
        delete h;
        return EDL_ENOMEM;
    }
    // a conv output feeding a batch norm must have no other consumer (its gradient is written, not added)
    h->arena = (char*)dev_arena;
    h->st = (hipStream_t)hip_stream;
    h->readers.assign(h->g.tensors.size(), 0);
    h->written.assign(h->g.tensors.size(), 0);
    h->op_done.assign(h->g.ops.size(), 0);
    h->grad_alias.assign(h->g.tensors.size(), nullptr);
    h->shard_n.reserve(kMaxP);
    h->perm.reserve((size_t)cfg->N);
    h->first_reader.assign(h->g.tensors.size(), -1);
    for (size_t i = 0; i < h->g.ops.size(); ++i) {
        const Op& op = h->g.ops[i];
        auto reads = [&](int t) {
            const size_t sx = (size_t)storage_of(h->g, t);
            h->readers[sx] += 1;
            if (h->first_reader[sx] < 0) h->first_reader[sx] = (int)i;
        };
        if (op.x >= 0) reads(op.x);
        if (op.kind == OP_BN && op.res >= 0) reads(op.res);
    }
    h->applied_from = h->g.P;
    rc = init_device_state(h);
    if (rc) {                            // whatever was created so far goes again
        destroy_handle(h);
        return rc;
    }
    *out = h;
    return EDL_OK;
}

// Pinned staging, events, the library's own side streams, and the initial model on the device.
static int init_device_state(edl_handle* h) {
    const edl_config* cfg = &h->cfg;
    const uint64_t seed = h->seed;
    for (int s = 0; s < kIdxSlots; ++s) {
        HIP_TRY(hipHostMalloc((void**)&h->idx_host[s], sizeof(int64_t) * (size_t)cfg->B, hipHostMallocDefault));
        HIP_TRY(hipEventCreateWithFlags(&h->idx_event[s], hipEventDisableTiming));
    }
    HIP_TRY(hipHostMalloc((void**)&h->loss_host, sizeof(float) * kMaxP, hipHostMallocDefault));
    // this GPU's copy of the static scratch buffer: its address is looked up once, with the device current
    HIP_TRY(hipGetDevice(&h->device));
    if (h->device >= 0 && h->device < kMaxDevices && g_static_scratch[h->device] == nullptr) {
        void* ptr = nullptr;
        HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        g_static_scratch[h->device] = ptr;
    }
    if (tune().wgrad_stream != 0) {
        HIP_TRY(hipStreamCreateWithFlags(&h->side, hipStreamNonBlocking));
        h->own_streams = true;
        HIP_TRY(hipStreamCreateWithFlags(&h->upd, hipStreamNonBlocking));
        const int rc = create_side_events(h);
        if (rc) return rc;
    }
    std::vector<float> init((size_t)h->g.P);
    std::vector<TransposeEntry> tab, tabv;
    // the copies below read these host arrays: whichever way this function is left, the stream is drained first
    struct DrainOnExit { hipStream_t st; ~DrainOnExit() { (void)hipStreamSynchronize(st); } } drain{h->st};
    he_init(h->g, seed, init.data());
    HIP_TRY(hipMemcpyAsync(h->w(), init.data(), sizeof(float) * (size_t)h->g.P, hipMemcpyHostToDevice, h->st));
    launch_fill_f32(h->v(), 0.f, h->g.P, h->st);
    if (h->adam()) launch_fill_f32(h->s2(), 0.f, h->g.P, h->st);
    for (const Op& op : h->g.ops)
        if (op.kind == OP_BN) {
            launch_fill_f32(h->running() + op.run_off, 0.f, op.K, h->st);
            launch_fill_f32(h->running() + op.run_off + op.K, 1.f, op.K, h->st);
        }
    {
        // bf16 layers of vector-friendly shape are transposed from the bf16 copy of the weights in 64x64
        // tiles; the others element by element from the float32 weights
        const double esz = cfg->dtype == EDL_DTYPE_BF16 ? 2.0 : 4.0;
        for (size_t i = 0; i < h->g.ops.size(); ++i) {
            const Op& op = h->g.ops[i];
            if (op.kind != OP_CONV || h->L.wT[i] < 0) continue;
            const Tensor& tx = h->g.tensors[(size_t)op.x];
            TransposeEntry te;
            te.src_off = op.w_off; te.dst_off = h->L.wT[i];
            te.K = op.K; te.RS = op.R * op.S; te.C = tx.C;
            if (cfg->dtype == EDL_DTYPE_BF16 && te.K % 8 == 0 && te.C % 8 == 0 && op.w_off % 8 == 0) {
                te.tile_start = h->tv_tiles;
                h->tv_tiles += ((te.C + 63) / 64) * ((te.K + 63) / 64) * te.RS;
                h->tv_bytes += 4.0 * (double)te.K * te.RS * te.C;
                tabv.push_back(te);
            } else {
                te.tile_start = h->t_tiles;
                h->t_tiles += ((te.C + 31) / 32) * ((te.K + 31) / 32) * te.RS;
                h->t_bytes += (4.0 + esz) * (double)te.K * te.RS * te.C;
                tab.push_back(te);
            }
        }
        h->t_entries = (int)tab.size();
        h->tv_entries = (int)tabv.size();
        if (!tab.empty())
            HIP_TRY(hipMemcpyAsync(h->at<TransposeEntry>(h->L.ttable), tab.data(), sizeof(TransposeEntry) * tab.size(),
                                   hipMemcpyHostToDevice, h->st));
        if (!tabv.empty())
            HIP_TRY(hipMemcpyAsync(h->at<TransposeEntry>(h->L.ttable) + h->g.ops.size(), tabv.data(),
                                   sizeof(TransposeEntry) * tabv.size(), hipMemcpyHostToDevice, h->st));
        HIP_TRY(hipStreamSynchronize(h->st));
    }
    h->weights_dirty = true;
    HIP_TRY(hipGetLastError());
    return EDL_OK;
}

int32_t edl_set_side_streams(edl_handle* h, void* wgrad_stream, void* update_stream) {
    if (!h) { set_error("null handle"); return EDL_EINVAL; }
    if ((wgrad_stream == nullptr) != (update_stream == nullptr)) { set_error("give both streams or neither"); return EDL_EINVAL; }
    if (wgrad_stream != nullptr && (wgrad_stream == update_stream || wgrad_stream == (void*)h->st || update_stream == (void*)h->st)) {
        set_error("the two side streams must differ from each other and from the job's stream");
        return EDL_EINVAL;
    }
    HIP_TRY(hipStreamSynchronize(h->st));
    release_side_streams(h);
    if (wgrad_stream == nullptr) return EDL_OK;         // everything on the job's stream from now on
    h->side = (hipStream_t)wgrad_stream;
    h->upd = (hipStream_t)update_stream;
    h->own_streams = false;
    const int rc = create_side_events(h);
    if (rc) { release_side_streams(h); return rc; }
    return EDL_OK;
}

int32_t edl_set_option(const char* name, int64_t value) {
    if (!tune_set(name, value)) { set_error("no option named '%s'", name ? name : "(null)"); return EDL_EINVAL; }
    return EDL_OK;
}

int32_t edl_get_option(const char* name, int64_t* out_value) {
    if (!tune_get(name, out_value)) { set_error("no option named '%s'", name ? name : "(null)"); return EDL_EINVAL; }
    return EDL_OK;
}

int32_t edl_bind_dataset(edl_handle* h, const float* dev_x, const int32_t* dev_y, int64_t N) {
    if (!h || !dev_x || !dev_y) { set_error("null argument"); return EDL_EINVAL; }
    if (N != h->cfg.N) { set_error("data set has %lld samples, the job was created for %lld", (long long)N, (long long)h->cfg.N); return EDL_EINVAL; }
    h->data_x = dev_x;
    h->data_y = dev_y;
    return EDL_OK;
}

int32_t edl_shard(const edl_handle* h, int64_t B, int32_t p, int64_t epoch, int64_t step_in_epoch, int64_t* out_idx,
                  int64_t* out_off) {
    if (!h) { set_error("null handle"); return EDL_EINVAL; }
    return edl_shard_host(h->seed, h->cfg.N, B, p, epoch, step_in_epoch, out_idx, out_off);
}

// forward + backward of one worker's shard: n samples whose indices are at
// dev_idx; gradient into G; mean loss into dev_loss[0]
// op_lo..op_hi: the slice of the layer list to run (the whole list in normal use;
// single layers from the debugging hooks, which then skip the gather)
static void forward_shard(edl_handle* h, const int64_t* dev_idx, int n, float* dev_loss, bool update_running,
                          size_t op_lo = 0, size_t op_hi = (size_t)-1) {
    const Graph& g = h->g;
    const int dt = h->cfg.dtype;
    hipStream_t st = h->st;
    const bool bf = dt == EDL_DTYPE_BF16;
    float* partial = h->sc<float>(h->L.partial);
    const Tensor& tin = g.tensors[0];
    if (dev_idx) {
        if (h->L.cpad != tin.C)
            launch_gather_pad(dt, h->data_x, h->data_y, dev_idx, n, (int64_t)tin.H * tin.W, tin.C, h->act(0),
                              h->at<int32_t>(h->L.labels), st);
        else
            launch_gather(dt, h->data_x, h->data_y, dev_idx, n, tin.elems(), h->act(0), h->at<int32_t>(h->L.labels), st);
    }
    if (op_hi > g.ops.size()) op_hi = g.ops.size();
    int stats_row_blocks = 0;   // > 0: the convolution just launched left the next batch norm's partial sums
    // the same for a convolution whose batch norm is not the next op: its sums wait in a buffer of their own
    float* const partial_held = h->sc<float>(h->L.partial_held);
    int held_rows = 0, held_tensor = -1;
    auto weights_of = [&](size_t i) {
        const Op& o = g.ops[i];
        const void* wsrc = bf ? (const void*)(h->at<uint16_t>(h->L.shadow) + o.w_off) : (const void*)(h->w() + o.w_off);
        if (h->L.wpad[i] >= 0) wsrc = h->arena + h->L.wpad[i];
        return wsrc;
    };
    // A residual block's projection shortcut (convolution + batch norm on the block's input) runs on the second
    // side stream while the main branch runs here; the block's last batch norm, which adds the two, waits for it.
    // Only when the whole list runs and nothing is being timed kernel by kernel.
    const bool branch = op_lo == 0 && op_hi == g.ops.size() && h->upd != nullptr && !prof_enabled() && tune().branch_stream != 0;
    std::vector<char>& done = h->op_done;
    std::fill(done.begin(), done.end(), 0);
    int join_tensor = -1;
    hipEvent_t join_event = nullptr;
    for (size_t i = op_lo; i < op_hi; ++i) {
        const Op& op = g.ops[i];
        if (done[i]) continue;
        if (branch && op.kind == OP_CONV && join_tensor < 0) {
            for (size_t j = i + 1; j + 2 < op_hi && j <= i + 8; ++j) {
                const Op& pj = g.ops[j];
                const Op& pb = g.ops[j + 1];
                if (!(pj.kind == OP_CONV && pj.x == op.x && pb.kind == OP_BN && pb.x == pj.y && pb.res < 0)) continue;
                bool joins = false;
                for (size_t k = j + 2; k < op_hi && k <= j + 3; ++k) joins = joins || (g.ops[k].kind == OP_BN && g.ops[k].res == pb.y);
                if (!joins) break;
                hipEvent_t go = h->ev_branch_go[h->branch_slot], dn = h->ev_branch_done[h->branch_slot];
                if (hipEventRecord(go, st) != hipSuccess || hipStreamWaitEvent(h->upd, go, 0) != hipSuccess) break;
                h->branch_slot = (h->branch_slot + 1) % kBranchEvents;
                float* const ps = h->sc<float>(h->L.partial_side);
                // this stream's own split-reduction scratch and wide-sums buffer (the main stream's are in use)
                const int rows = launch_conv_fwd(dt, geom_padded(g, pj, n, h->L.cpad), h->act(pj.x), weights_of(j),
                                                 pj.bias ? h->w() + pj.b_off : nullptr, pj.relu, g.tensors[(size_t)pj.y].fp32,
                                                 h->act(pj.y), h->sc<float>(h->L.splitk_side), (size_t)h->L.splitk_scratch_bytes, ps,
                                                 WideSums{h->sc<float>(h->L.wide_sums_side), (size_t)h->L.wide_sums_floats}, h->upd);
                const Tensor& t = g.tensors[(size_t)pb.x];
                launch_bn_forward(dt, h->act(pb.x), nullptr, h->act(pb.y), h->w() + pb.w_off, h->w() + pb.b_off,
                                  h->at<float>(h->L.bn_save[j + 1]), update_running ? h->running() + pb.run_off : nullptr,
                                  (int64_t)n * t.H * t.W, t.C, pb.relu, ps, rows, h->upd);
                (void)hipEventRecord(dn, h->upd);
                done[j] = done[j + 1] = 1;
                join_tensor = pb.y;
                join_event = dn;
                break;
            }
        }
        switch (op.kind) {
            case OP_CONV: {
                const void* wsrc = weights_of(i);
                // the batch norm that follows (in this call) can take its sums from the convolution's epilogue
                const bool bn_next = i + 1 < op_hi && g.ops[i + 1].kind == OP_BN && g.ops[i + 1].x == op.y;
                // ... or a later one of this call, if the held buffer is free
                const bool tune_held = tune().held_stats != 0;
                bool bn_later = false;
                if (!bn_next && tune_held && held_tensor < 0)
                    for (size_t j = i + 2; j < op_hi && j <= i + 4 && !bn_later; ++j)
                        bn_later = g.ops[j].kind == OP_BN && g.ops[j].x == op.y;
                const int rows = launch_conv_fwd(dt, geom_padded(g, op, n, h->L.cpad), h->act(op.x), wsrc,
                                                 op.bias ? h->w() + op.b_off : nullptr, op.relu, g.tensors[(size_t)op.y].fp32,
                                                 h->act(op.y), h->sc<float>(h->L.splitk_scratch),
                                                 (size_t)h->L.splitk_scratch_bytes,
                                                 bn_next ? partial : bn_later ? partial_held : nullptr,
                                                 WideSums{h->sc<float>(h->L.wide_sums), (size_t)h->L.wide_sums_floats}, st);
                if (bn_later) {
                    if (rows > 0) { held_rows = rows; held_tensor = op.y; }
                    stats_row_blocks = 0;
                } else {
                    stats_row_blocks = rows;
                }
                break;
            }
            case OP_BN: {
                const Tensor& t = g.tensors[(size_t)op.x];
                const bool held = held_tensor == op.x && held_rows > 0;
                if (op.res >= 0 && op.res == join_tensor) {      // the shortcut's part comes from the other stream
                    (void)hipStreamWaitEvent(st, join_event, 0);
                    join_tensor = -1;
                }
                launch_bn_forward(dt, h->act(op.x), op.res >= 0 ? h->act(op.res) : nullptr, h->act(op.y), h->w() + op.w_off,
                                  h->w() + op.b_off, h->at<float>(h->L.bn_save[i]),
                                  update_running ? h->running() + op.run_off : nullptr, (int64_t)n * t.H * t.W, t.C, op.relu,
                                  held ? partial_held : partial, held ? held_rows : stats_row_blocks, st);
                if (held) { held_rows = 0; held_tensor = -1; }
                stats_row_blocks = 0;
                break;
            }
            case OP_MAXPOOL: {
                const Tensor& tx = g.tensors[(size_t)op.x];
                const Tensor& ty = g.tensors[(size_t)op.y];
                launch_maxpool_forward(dt, h->act(op.x), h->act(op.y), h->at<uint8_t>(h->L.pool_arg[i]), n, tx.H, tx.W, tx.C,
                                       op.R, op.stride, op.pad, ty.H, ty.W, st);
                break;
            }
            case OP_GAVGPOOL: {
                const Tensor& tx = g.tensors[(size_t)op.x];
                launch_gavgpool_forward(dt, h->act(op.x), h->act(op.y), n, tx.H * tx.W, tx.C, st);
                break;
            }
            case OP_LOSS:
                launch_softmax_ce(dt, (const float*)h->act(op.x), h->at<int32_t>(h->L.labels), h->grad(op.x),
                                  h->sc<float>(h->L.row_loss), dev_loss, n, g.classes, st);
                break;
        }
    }
    if (join_tensor >= 0) (void)hipStreamWaitEvent(st, join_event, 0);   // a branch nobody joined (cannot happen)
}

static int apply_range(edl_handle* h, int32_t p, int64_t lo, int64_t hi, hipStream_t st, int max_blocks = 0);

// early_p > 0: this is the last backward pass of a step of early_p shards, so gradients that are final may be
// applied while the pass goes on.
// held (debugging hook only): tensors whose gradient buffers already hold a contribution the pass adds to.
static void backward_shard(edl_handle* h, int n, float* G, size_t op_lo = 0, size_t op_hi = (size_t)-1, int early_p = 0,
                           const std::vector<int>* held = nullptr) {
    const Graph& g = h->g;
    const int dt = h->cfg.dtype;
    hipStream_t st = h->st;
    float* partial = h->sc<float>(h->L.partial);
    float* coef = h->sc<float>(h->L.coef);
    if (h->transposes_pending) {          // the transposed weight copies were made on the weight-gradient stream
        (void)hipStreamWaitEvent(st, h->ev_tr_done, 0);
        h->transposes_pending = false;
    }
    std::vector<char>& written = h->written;     // sized at init: no allocation in the pass
    std::fill(written.begin(), written.end(), 0);
    std::fill(h->grad_alias.begin(), h->grad_alias.end(), nullptr);
    if (held)
        for (int t : *held) written[(size_t)storage_of(g, t)] = 1;
    if (op_hi > g.ops.size()) op_hi = g.ops.size();
    // per-kernel timing wants one kernel at a time
    const bool overlap = h->side != nullptr && !prof_enabled();
    bool used_side = false, used_upd = false;
    // the projection shortcut's backward on the second side stream (see forward_shard)
    const bool branch = overlap && op_lo == 0 && op_hi == g.ops.size() && h->upd != nullptr && tune().branch_stream != 0;
    std::vector<char>& done = h->op_done;
    std::fill(done.begin(), done.end(), 0);
    int join_storage = -1;               // gradient buffer the branch stream is still writing
    hipEvent_t join_event = nullptr;
    size_t fused_for = (size_t)-1;   // the layer whose masked gradient and column sums the dgrad after it left
    int fused_rows = 0;
    size_t premasked_for = (size_t)-1;   // the layer whose gradient the max pool after it left masked by its ReLU
    for (size_t ii = op_hi; ii-- > op_lo;) {
        const Op& op = g.ops[ii];
        if (done[ii]) continue;
        if (join_storage >= 0 && op.x >= 0 && storage_of(g, op.x) == join_storage) {
            // this layer adds to the gradient the branch stream has been writing
            (void)hipStreamWaitEvent(st, join_event, 0);
            join_storage = -1;
        }
        switch (op.kind) {
            case OP_LOSS:
                written[(size_t)storage_of(g, op.x)] = 1;
                break;
            case OP_CONV: {
                const ConvGeom q = geom_padded(g, op, n, h->L.cpad);
                const int64_t M = (int64_t)n * q.Ho * q.Wo;
                const bool padded = h->L.wpad[ii] >= 0;
                launch_bias_relu_backward(dt, h->act(op.y), h->grad(op.y), op.bias ? G + op.b_off : nullptr, M, op.K,
                                          op.relu && premasked_for != ii, partial, fused_for == ii ? fused_rows : 0, st);
                // The weight gradient needs only dy (final from here on) and the layer's input, and nothing
                // before the update reads it: it runs on the second stream, beside the chain of input
                // gradients, whose short kernels leave part of the chip idle.
                hipStream_t ws = st;
                // The first layers' weight gradients are the last of the pass: by then the main stream has nothing
                // else to do, so they stay on it (with a scratch of their own) and run beside the second stream's backlog.
                const int tail_main = (int)tune().wgrad_tail_main;
                int conv_ordinal = 0;
                for (size_t j = 0; j < ii; ++j) conv_ordinal += g.ops[j].kind == OP_CONV;
                const bool on_main = overlap && conv_ordinal < tail_main;
                float* const wscratch = h->sc<float>(on_main ? h->L.wgrad_scratch2 : h->L.wgrad_scratch);
                if (overlap && !on_main) {
                    hipEvent_t ev = h->ev_ready[h->ev_slot];
                    h->ev_slot = (h->ev_slot + 1) % kReadyEvents;
                    if (hipEventRecord(ev, st) == hipSuccess && hipStreamWaitEvent(h->side, ev, 0) == hipSuccess) {
                        ws = h->side;
                        used_side = true;
                    }
                }
                launch_conv_wgrad(dt, q, h->act(op.x), h->grad(op.y), padded ? h->sc<float>(h->L.dwpad) : G + op.w_off,
                                  wscratch, (size_t)h->L.wgrad_scratch_bytes, ws);
                if (padded)
                    launch_unpad_rows(h->sc<float>(h->L.dwpad), G + op.w_off, (int64_t)op.K * op.R * op.S, g.tensors[0].C, h->L.cpad, ws);
                // Parameters are laid out in layer order, so everything from this layer's weights on now has its
                // final gradient: the second stream holds the weight gradients, and the event it waited for
                // covers what the main stream has written (bias and batch-norm gradients of the later layers)
                // and read (their batch-norm scales).  Nothing of the rest of the pass reads those parameters
                // (input gradients use the transposed copies), so their update starts now, on a third stream, if
                // the layer is a large one (chunk_min weights or more: the update of a small piece gains less than
                // its launch beside the input-gradient chain costs).  The piece starts at the layer's first weight
                // rounded up to 64, so that the vector accesses stay aligned; the few weights below go with the
                // next piece or with the rest of the update after the pass.
                const int64_t chunk_min = tune().early_update;
                if (early_p > 0 && ws == h->side && ws != st && h->upd != nullptr && chunk_min > 0) {
                    const int64_t lo = (op.w_off + 63) / 64 * 64;
                    const int64_t own = (int64_t)op.K * op.R * op.S * g.tensors[(size_t)op.x].C;
                    if (lo > 0 && lo < h->applied_from && own >= chunk_min) {
                        hipEvent_t ev = h->ev_chunk[h->chunk_slot];
                        h->chunk_slot = (h->chunk_slot + 1) % kChunkEvents;
                        if (hipEventRecord(ev, h->side) == hipSuccess && hipStreamWaitEvent(h->upd, ev, 0) == hipSuccess) {
                            // held to few workgroups: a full-width launch would take the CUs from the chain of
                            // input gradients for as long as it runs
                            const int early_blocks = (int)tune().early_blocks;
                            apply_range(h, early_p, lo, h->applied_from, h->upd, early_blocks);
                            h->applied_from = lo;
                            used_upd = true;
                        }
                    }
                }
                const int sx = storage_of(g, op.x);
                if (sx != 0) {
                    // If the layer just before in the list produced this convolution's input and ends in a ReLU, and
                    // this convolution is the first reader of that tensor in the list (so every other reader, such as
                    // the shortcut of a residual block, has already added its part), that layer's backward starts with
                    // the masked gradient and its column sums: the dgrad's epilogue can leave both (see DgradMask),
                    // and that layer then skips its own reduction pass.
                    DgradMask mask = {};
                    const bool acc = written[(size_t)sx] != 0;
                    const bool fuse_joins = tune().fused_mask_join != 0;
                    const bool last_writer = h->first_reader[(size_t)sx] == ii &&
                                             (h->readers[(size_t)sx] == 1 ? !acc : (fuse_joins && acc));
                    if (ii > op_lo && last_writer) {
                        const Op& prod = g.ops[ii - 1];
                        if (prod.relu && storage_of(g, prod.y) == sx && (prod.kind == OP_BN || prod.kind == OP_CONV)) {
                            mask.act = h->act(op.x);
                            mask.sums = partial;
                            mask.wide = WideSums{h->sc<float>(h->L.wide_sums), (size_t)h->L.wide_sums_floats};
                            if (prod.kind == OP_BN) {
                                mask.xin = h->act(prod.x);
                                mask.mean_rstd = h->at<float>(h->L.bn_save[ii - 1]);
                            }
                        }
                    }
                    const int rows = launch_conv_dgrad(dt, q, h->grad(op.y), h->arena + h->L.wT[ii], acc, h->grad(op.x),
                                                       h->sc<float>(h->L.splitk_scratch), (size_t)h->L.splitk_scratch_bytes,
                                                       mask.act ? &mask : nullptr, st, acc ? h->grad_alias[(size_t)sx] : nullptr);
                    h->grad_alias[(size_t)sx] = nullptr;
                    if (rows > 0) { fused_for = ii - 1; fused_rows = rows; }
                    written[(size_t)sx] = 1;
                }
                break;
            }
            case OP_BN: {
                const Tensor& t = g.tensors[(size_t)op.x];
                const int sx = storage_of(g, op.x);
                void* dres = nullptr;
                bool dres_acc = false;
                if (op.res >= 0 && storage_of(g, op.res) != 0) {
                    const int sr = storage_of(g, op.res);
                    dres = h->grad(op.res);
                    dres_acc = written[(size_t)sr] != 0;
                    written[(size_t)sr] = 1;
                    // An identity shortcut whose gradient would be a plain copy of this layer's (already masked)
                    // output gradient: nothing is copied; the one other reader of the tensor - a stride-1
                    // convolution later in this pass, which adds its part - reads it from where it lies.
                    const bool dy_is_dres = !dres_acc && (!op.relu || fused_for == ii || premasked_for == ii);
                    const int fr = h->first_reader[(size_t)sr];
                    if (dy_is_dres && tune().alias_shortcut != 0 && h->readers[(size_t)sr] == 2 && fr >= (int)op_lo && fr < (int)ii &&
                        g.ops[(size_t)fr].kind == OP_CONV && g.ops[(size_t)fr].stride == 1 && storage_of(g, g.ops[(size_t)fr].x) == sr) {
                        h->grad_alias[(size_t)sr] = h->grad(op.y);
                        dres = nullptr;
                    }
                    // The same for a projection shortcut: the batch norm listed just before produced the tensor and is
                    // its only other user, and its backward only reads the gradient.
                    if (dy_is_dres && tune().alias_shortcut != 0 && h->readers[(size_t)sr] == 1 && ii >= op_lo + 1 &&
                        g.ops[ii - 1].kind == OP_BN && g.ops[ii - 1].y == op.res && !g.ops[ii - 1].relu) {
                        h->grad_alias[(size_t)sr] = h->grad(op.y);
                        dres = nullptr;
                    }
                }
                const size_t sy = (size_t)storage_of(g, op.y);
                const void* const dy_src = h->grad_alias[sy] ? h->grad_alias[sy] : h->grad(op.y);
                h->grad_alias[sy] = nullptr;
                launch_bn_backward(dt, h->act(op.x), h->act(op.y), dy_src, h->grad(op.x), dres, dres_acc,
                                   h->w() + op.w_off, h->at<float>(h->L.bn_save[ii]), G + op.w_off, G + op.b_off,
                                   (int64_t)n * t.H * t.W, t.C, op.relu && premasked_for != ii, partial, coef,
                                   fused_for == ii ? fused_rows : 0, st);
                written[(size_t)sx] = 1;
                // The gradient of the shortcut is final now.  If the shortcut is a projection (the convolution and
                // batch norm listed just before), its backward - batch norm, weight gradient, input gradient into
                // the block's input - needs nothing else of the main branch: it goes to the second side stream,
                // with a reduction scratch of its own, while the main branch's chain continues here.  The block's
                // first convolution, which adds to the same input gradient, waits for it.
                if (branch && op.res >= 0 && ii >= op_lo + 2 && join_storage < 0) {
                    const Op& pb = g.ops[ii - 1];
                    const Op& pj = g.ops[ii - 2];
                    const int pj_sx = pj.x >= 0 ? storage_of(g, pj.x) : 0;
                    if (pb.kind == OP_BN && pb.y == op.res && pb.res < 0 && pj.kind == OP_CONV && pj.y == pb.x && pj_sx != 0 &&
                        h->L.wpad[ii - 2] < 0) {
                        hipEvent_t go = h->ev_branch_go[h->branch_slot], dn = h->ev_branch_done[h->branch_slot];
                        hipEvent_t wg = h->ev_ready[h->ev_slot];
                        if (hipEventRecord(go, st) == hipSuccess && hipStreamWaitEvent(h->upd, go, 0) == hipSuccess) {
                            h->branch_slot = (h->branch_slot + 1) % kBranchEvents;
                            h->ev_slot = (h->ev_slot + 1) % kReadyEvents;
                            hipStream_t bs = h->upd;
                            float* const ps = h->sc<float>(h->L.partial_side);
                            const Tensor& tb = g.tensors[(size_t)pb.x];
                            const size_t spy = (size_t)storage_of(g, pb.y);
                            const void* const pdy = h->grad_alias[spy] ? h->grad_alias[spy] : h->grad(pb.y);
                            h->grad_alias[spy] = nullptr;
                            launch_bn_backward(dt, h->act(pb.x), h->act(pb.y), pdy, h->grad(pb.x), nullptr, false,
                                               h->w() + pb.w_off, h->at<float>(h->L.bn_save[ii - 1]), G + pb.w_off, G + pb.b_off,
                                               (int64_t)n * tb.H * tb.W, tb.C, pb.relu, ps, h->sc<float>(h->L.coef_side), 0, bs);
                            written[(size_t)storage_of(g, pb.x)] = 1;
                            const ConvGeom qj = geom_padded(g, pj, n, h->L.cpad);
                            launch_bias_relu_backward(dt, h->act(pj.y), h->grad(pj.y), pj.bias ? G + pj.b_off : nullptr,
                                                      (int64_t)n * qj.Ho * qj.Wo, pj.K, pj.relu, ps, 0, bs);
                            // weight gradient: on the first side stream like every other, behind this stream's work
                            hipStream_t ws = bs;
                            if (hipEventRecord(wg, bs) == hipSuccess && hipStreamWaitEvent(h->side, wg, 0) == hipSuccess) {
                                ws = h->side;
                                used_side = true;
                            }
                            launch_conv_wgrad(dt, qj, h->act(pj.x), h->grad(pj.y), G + pj.w_off,
                                              ws == h->side ? h->sc<float>(h->L.wgrad_scratch) : nullptr,
                                              ws == h->side ? (size_t)h->L.wgrad_scratch_bytes : 0, ws);
                            // input gradient, with this stream's own split-reduction scratch; nothing to hand over (the
                            // block's first convolution is the last to add to this gradient)
                            launch_conv_dgrad(dt, qj, h->grad(pj.y), h->arena + h->L.wT[ii - 2], written[(size_t)pj_sx] != 0,
                                              h->grad(pj.x), h->sc<float>(h->L.splitk_side), (size_t)h->L.splitk_scratch_bytes, nullptr, bs);
                            written[(size_t)pj_sx] = 1;
                            (void)hipEventRecord(dn, bs);
                            done[ii - 1] = done[ii - 2] = 1;
                            join_storage = pj_sx;
                            join_event = dn;
                            used_upd = true;
                        }
                    }
                }
                break;
            }
            case OP_MAXPOOL: {
                const Tensor& tx = g.tensors[(size_t)op.x];
                const Tensor& ty = g.tensors[(size_t)op.y];
                const int sx = storage_of(g, op.x);
                if (sx != 0) {
                    // a ReLU layer just before in the list whose output only this pool reads: its gradient can leave
                    // the pool already masked
                    const void* relu_act = nullptr;
                    if (ii > op_lo && written[(size_t)sx] == 0 && h->readers[(size_t)sx] == 1) {
                        const Op& prod = g.ops[ii - 1];
                        if (prod.relu && storage_of(g, prod.y) == sx && (prod.kind == OP_BN || prod.kind == OP_CONV))
                            relu_act = h->act(op.x);
                    }
                    if (launch_maxpool_backward(dt, h->grad(op.y), h->at<uint8_t>(h->L.pool_arg[ii]), h->grad(op.x),
                                                written[(size_t)sx] != 0, n, tx.H, tx.W, tx.C, op.R, op.stride, op.pad, ty.H,
                                                ty.W, relu_act, st))
                        premasked_for = ii - 1;
                    written[(size_t)sx] = 1;
                }
                break;
            }
            case OP_GAVGPOOL: {
                const Tensor& tx = g.tensors[(size_t)op.x];
                const int sx = storage_of(g, op.x);
                if (sx != 0) {
                    launch_gavgpool_backward(dt, h->grad(op.y), h->grad(op.x), written[(size_t)sx] != 0, n, tx.H * tx.W, tx.C, st);
                    written[(size_t)sx] = 1;
                }
                break;
            }
        }
    }
    // the next forward pass overwrites the activations the weight gradients read, and the update reads G
    if (used_side) {
        (void)hipEventRecord(h->ev_side_done, h->side);
        (void)hipStreamWaitEvent(st, h->ev_side_done, 0);
    }
    if (used_upd) {
        (void)hipEventRecord(h->ev_upd_done, h->upd);
        (void)hipStreamWaitEvent(st, h->ev_upd_done, 0);
    }
}

static int check_p(const edl_handle* h, int32_t p) {
    if (p <= 0 || p > h->cfg.p_max) { set_error("p=%d outside [1, p_max=%d]", p, h->cfg.p_max); return EDL_EINVAL; }
    if (h->cfg.B % p) { set_error("B=%lld is not a multiple of p=%d", (long long)h->cfg.B, p); return EDL_EINDIVISIBLE; }
    if (h->cfg.B / p > h->cfg.max_shard) { set_error("shard of %lld samples exceeds max_shard=%d", (long long)(h->cfg.B / p), h->cfg.max_shard); return EDL_ENOMEM; }
    return EDL_OK;
}

int32_t edl_gradients(edl_handle* h, int32_t p, const int64_t* idx, const int64_t* off, float* out_loss) {
    if (!h) { set_error("null handle"); return EDL_EINVAL; }
    if (!h->data_x) { set_error("no data set bound"); return EDL_EINVAL; }
    if ((idx == nullptr) != (off == nullptr)) { set_error("idx and off must both be given or both be NULL"); return EDL_EINVAL; }
    const int64_t B = h->cfg.B;
    int64_t sizes[kMaxP];
    if (idx) {
        // the caller's cut of the mini-batch: any shard sizes that fit the workspace (equal ones in normal use)
        if (p <= 0 || p > h->cfg.p_max) { set_error("p=%d outside [1, p_max=%d]", p, h->cfg.p_max); return EDL_EINVAL; }
        if (off[0] != 0 || off[p] != B) { set_error("off must run from 0 to B=%lld", (long long)B); return EDL_ERANGE; }
        for (int k = 0; k < p; ++k) {
            const int64_t nk = off[k + 1] - off[k];
            if (nk < 0) { set_error("off[%d] > off[%d]", k, k + 1); return EDL_ERANGE; }
            if (nk > h->cfg.max_shard) { set_error("shard %d of %lld samples exceeds max_shard=%d", k, (long long)nk, h->cfg.max_shard); return EDL_ENOMEM; }
            sizes[k] = nk;
        }
    } else {
        const int rc = check_p(h, p);
        if (rc) return rc;
        for (int k = 0; k < p; ++k) sizes[k] = B / p;
    }
    bool equal = true;
    for (int k = 0; k < p; ++k) equal = equal && sizes[k] == sizes[0];
    const int slot = h->idx_slot;
    h->idx_slot = (slot + 1) % kIdxSlots;
    HIP_TRY(hipEventSynchronize(h->idx_event[slot]));
    int64_t* stage = h->idx_host[slot];
    if (idx) {
        for (int64_t i = 0; i < B; ++i) {
            if (idx[i] < 0 || idx[i] >= h->cfg.N) { set_error("idx[%lld]=%lld outside [0,N)", (long long)i, (long long)idx[i]); return EDL_ERANGE; }
            stage[i] = idx[i];
        }
    } else {
        if (h->perm_epoch != h->prog.epoch) {
            epoch_permutation(h->seed, h->prog.epoch, h->cfg.N, h->perm);
            h->perm_epoch = h->prog.epoch;
        }
        memcpy(stage, h->perm.data() + h->prog.step_in_epoch * B, sizeof(int64_t) * (size_t)B);
    }
    h->shard_n.assign(sizes, sizes + p);
    h->shards_equal = equal;
    int64_t* dev_idx = h->at<int64_t>(h->L.idx);
    HIP_TRY(hipMemcpyAsync(dev_idx, stage, sizeof(int64_t) * (size_t)B, hipMemcpyHostToDevice, h->st));
    HIP_TRY(hipEventRecord(h->idx_event[slot], h->st));
    if (h->weights_dirty) {
        refresh_weight_copies(h);
        h->weights_dirty = false;
    }
    // The transposed copies are first read by the backward pass: they are made on the weight-gradient stream, which
    // is idle during the forward pass, and the first backward pass waits for them.
    h->transposes_pending = false;
    if (h->side != nullptr && !prof_enabled() && tune().transpose_stream != 0 &&
        hipEventRecord(h->ev_tr_go, h->st) == hipSuccess && hipStreamWaitEvent(h->side, h->ev_tr_go, 0) == hipSuccess) {
        transpose_weights(h, h->side);
        h->transposes_pending = hipEventRecord(h->ev_tr_done, h->side) == hipSuccess;
        if (!h->transposes_pending) (void)hipStreamSynchronize(h->side);
    } else {
        transpose_weights(h, h->st);
    }
    float* dev_losses = h->at<float>(h->L.losses);
    int64_t at = 0;
    bool first = true;       // the first worker that has samples keeps the running statistics
    int last_k = -1;
    for (int k = 0; k < p; ++k)
        if (sizes[k] > 0) last_k = k;
    for (int k = 0; k < p; ++k) {
        const int64_t nk = sizes[k];
        if (nk > 0) {
            forward_shard(h, dev_idx + at, (int)nk, dev_losses + k, first);
            backward_shard(h, (int)nk, h->grad_buf(k), 0, (size_t)-1, k == last_k ? h->early_p : 0);
            first = false;
        }
        at += nk;
    }
    HIP_TRY(hipGetLastError());
    if (out_loss) {
        HIP_TRY(hipMemcpyAsync(h->loss_host, dev_losses, sizeof(float) * (size_t)p, hipMemcpyDeviceToHost, h->st));
        HIP_TRY(hipStreamSynchronize(h->st));
        double s = 0;
        if (equal) {
            for (int k = 0; k < p; ++k) s += h->loss_host[k];
            s /= p;
        } else {   // the mean over the mini-batch: every worker's mean weighs in with its share
            for (int k = 0; k < p; ++k)
                if (sizes[k] > 0) s += (double)h->loss_host[k] * ((double)sizes[k] / (double)B);
        }
        *out_loss = (float)s;
    }
    h->grads_pending = true;
    return EDL_OK;
}

// bias corrections of update number t, formed in double
static void adam_corrections(double beta1, double beta2, int64_t t, float* c1, float* c2) {
    *c1 = (float)(1.0 / (1.0 - std::pow(beta1, (double)t)));
    *c2 = (float)(1.0 / (1.0 - std::pow(beta2, (double)t)));
}

// The update of parameters [lo, hi) from the gradient buffers of the step's p shards (every buffer weighs in
// with its shard's share of the mini-batch if the shards are unequal), on stream st.  lo is a multiple of 4.
static int apply_range(edl_handle* h, int32_t p, int64_t lo, int64_t hi, hipStream_t st, int max_blocks) {
    if (hi <= lo) return EDL_OK;
    uint16_t* shadow = h->cfg.dtype == EDL_DTYPE_BF16 ? h->at<uint16_t>(h->L.shadow) + lo : nullptr;
    const int64_t len = hi - lo;
    GradPtrs gp = {};
    ShardShares sh = {};
    int np = 0;
    if (h->shards_equal) {
        for (int k = 0; k < p; ++k) gp.g[k] = h->grad_buf(k) + lo;
        np = p;
    } else {
        for (int k = 0; k < p; ++k) {
            if (h->shard_n[(size_t)k] == 0) continue;
            gp.g[np] = h->grad_buf(k) + lo;
            sh.share[np] = (float)((double)h->shard_n[(size_t)k] / (double)h->cfg.B);
            ++np;
        }
    }
    if (h->adam()) {
        float c1, c2;
        adam_corrections(h->cfg.momentum, h->cfg.beta2, h->prog.step + 1, &c1, &c2);
        launch_adam_update(np, gp, h->shards_equal ? nullptr : &sh, h->w() + lo, h->v() + lo, h->s2() + lo, shadow, len, h->cfg.lr,
                           h->cfg.momentum, h->cfg.beta2, h->cfg.eps, h->cfg.wd, c1, c2, st, max_blocks);
    } else if (h->shards_equal) {
        launch_average_update(np, gp, h->w() + lo, h->v() + lo, shadow, len, h->cfg.lr, h->cfg.momentum, h->cfg.wd, st, max_blocks);
    } else {
        launch_weighted_update(np, gp, sh, h->w() + lo, h->v() + lo, shadow, len, h->cfg.lr, h->cfg.momentum, h->cfg.wd, st);
    }
    return EDL_OK;
}

int32_t edl_apply(edl_handle* h, int32_t p) {
    if (!h) { set_error("null handle"); return EDL_EINVAL; }
    // the gradient buffers are applied once: a second call, or one without gradients, would move the model by
    // whatever the buffers happen to hold
    if (!h->grads_pending) { set_error("no gradients pending: edl_apply follows one edl_gradients"); return EDL_EINVAL; }
    if ((size_t)p != h->shard_n.size()) {
        set_error("p=%d, but the pending gradients are of %zu shards", p, h->shard_n.size());
        return EDL_EINVAL;
    }
    h->grads_pending = false;
    // what the backward pass has not already updated (all of it, unless this is the second half of edl_step)
    apply_range(h, p, 0, h->applied_from, h->st);
    h->applied_from = h->g.P;
    HIP_TRY(hipGetLastError());
    h->prog.step += 1;
    h->prog.step_in_epoch += 1;
    if (h->prog.step_in_epoch == h->cfg.N / h->cfg.B) {
        h->prog.step_in_epoch = 0;
        h->prog.epoch += 1;
    }
    return EDL_OK;
}

int32_t edl_step(edl_handle* h, int32_t p, const int64_t* idx, const int64_t* off, float* out_loss) {
    if (h) h->early_p = p;      // the last backward pass may start the update
    const int rc = edl_gradients(h, p, idx, off, out_loss);
    if (h) h->early_p = 0;
    if (rc) {
        if (h && h->applied_from != h->g.P) {   // cannot happen after the arguments passed their checks
            set_error("the step failed after part of the update was launched");
            h->applied_from = h->g.P;
        }
        return rc;
    }
    return edl_apply(h, p);
}

int32_t edl_step_static_scratch(edl_handle* h, int32_t p, const int64_t* idx, const int64_t* off, float* out_loss) {
    if (!h) { set_error("null handle"); return EDL_EINVAL; }
    const int64_t need = h->L.scratch_hi - h->L.scratch_lo;
    if (need > (int64_t)EDL_STATIC_SCRATCH_BYTES) {
        set_error("the kernels of this job need %lld bytes of scratch; the static buffer holds %lld (use edl_step, whose "
                  "scratch is part of the caller's arena)", (long long)need, (long long)EDL_STATIC_SCRATCH_BYTES);
        return EDL_ENOMEM;
    }
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev != h->device || dev < 0 || dev >= kMaxDevices || g_static_scratch[dev] == nullptr) {
        set_error("device %d is current, the job was created on device %d (or its static scratch was never set up)", dev, h->device);
        return EDL_EINVAL;
    }
    // nothing in the buffer has to start at zero: every partial result is written by the launch that precedes its
    // reader (the arena's piece is never cleared either)
    h->scratch_base = (char*)g_static_scratch[dev];
    const int rc = edl_step(h, p, idx, off, out_loss);
    h->scratch_base = nullptr;
    return rc;
}

int32_t edl_profile_parallelism(edl_handle* h, int32_t min_p, int32_t max_p, int32_t steps, edl_parallelism_point* out,
                                int32_t cap, int32_t* out_count) {
    if (!h || !out || !out_count) { set_error("null argument"); return EDL_EINVAL; }
    *out_count = 0;
    if (steps <= 0 || steps > 256) { set_error("steps=%d outside [1, 256]", steps); return EDL_EINVAL; }
    if (!h->data_x) { set_error("no data set bound"); return EDL_EINVAL; }
    std::vector<int32_t> ps;
    for (int32_t p = std::min(max_p, h->cfg.p_max); p >= std::max(min_p, 1); --p)
        if (h->cfg.B % p == 0 && h->cfg.B / p <= h->cfg.max_shard) ps.push_back(p);
    if (ps.empty()) { set_error("no parallelism in [%d, %d] fits B=%lld, p_max=%d, max_shard=%d", min_p, max_p, (long long)h->cfg.B, h->cfg.p_max, h->cfg.max_shard); return EDL_EINVAL; }
    if ((size_t)cap < ps.size()) { set_error("%zu entries needed", ps.size()); return EDL_ENOMEM; }
    std::vector<hipEvent_t> ev((size_t)steps * 2 + 1);
    for (hipEvent_t& e : ev) HIP_TRY(hipEventCreate(&e));
    int rc = EDL_OK;
    for (size_t i = 0; i < ps.size() && rc == EDL_OK; ++i) {
        const int32_t p = ps[i];
        // ev[2t]: before the gradient passes of step t; ev[2t+1]: after them, before the update; ev[2*steps]: end
        for (int t = 0; t < steps && rc == EDL_OK; ++t) {
            if (hipEventRecord(ev[(size_t)2 * t], h->st) != hipSuccess) { set_error("hipEventRecord failed"); rc = EDL_EHIP; break; }
            rc = edl_gradients(h, p, nullptr, nullptr, nullptr);
            if (rc) break;
            if (hipEventRecord(ev[(size_t)2 * t + 1], h->st) != hipSuccess) { set_error("hipEventRecord failed"); rc = EDL_EHIP; break; }
            rc = edl_apply(h, p);
        }
        if (rc) break;
        if (hipEventRecord(ev[(size_t)2 * steps], h->st) != hipSuccess || hipEventSynchronize(ev[(size_t)2 * steps]) != hipSuccess) {
            set_error("timing events failed");
            rc = EDL_EHIP;
            break;
        }
        float total_ms = 0.f;
        double grad_ms = 0.0;
        (void)hipEventElapsedTime(&total_ms, ev[0], ev[(size_t)2 * steps]);
        for (int t = 0; t < steps; ++t) {
            float ms = 0.f;
            (void)hipEventElapsedTime(&ms, ev[(size_t)2 * t], ev[(size_t)2 * t + 1]);
            grad_ms += ms;
        }
        edl_parallelism_point& o = out[i];
        o.p = p;
        o.shard = (int32_t)(h->cfg.B / p);
        o.ms_per_step = (double)total_ms / steps;
        o.samples_per_s = (double)h->cfg.B / (o.ms_per_step * 1e-3);
        o.worker_samples_per_s = (double)h->cfg.B / (grad_ms / steps * 1e-3);
        o.efficiency = 0.0;
    }
    for (hipEvent_t e : ev) (void)hipEventDestroy(e);
    if (rc) return rc;
    double best = 0.0;
    for (size_t i = 0; i < ps.size(); ++i) best = std::max(best, out[i].worker_samples_per_s);
    for (size_t i = 0; i < ps.size(); ++i) out[i].efficiency = best > 0 ? out[i].worker_samples_per_s / best : 0.0;
    *out_count = (int32_t)ps.size();
    return EDL_OK;
}

int32_t edl_snapshot(edl_handle* h, void* dev_dst, size_t cap, size_t* out_written) {
    if (!h || !dev_dst) { set_error("null argument"); return EDL_EINVAL; }
    const int64_t P = h->g.P, R = h->g.R;
    const size_t need = EDL_SNAPSHOT_HEADER_BYTES + 4 * (size_t)h->state_floats();
    if (cap < need) { set_error("snapshot needs %zu bytes, buffer has %zu", need, cap); return EDL_ENOMEM; }
    alignas(8) char hdr[EDL_SNAPSHOT_HEADER_BYTES];
    memset(hdr, 0, sizeof(hdr));
    SnapshotHeader sh = {};
    sh.magic = EDL_SNAPSHOT_MAGIC; sh.version = 1; sh.model = (uint32_t)h->cfg.model; sh.dtype = (uint32_t)h->cfg.dtype;
    sh.seed = h->seed; sh.N = h->cfg.N; sh.B = h->cfg.B;
    sh.step = h->prog.step; sh.epoch = h->prog.epoch; sh.step_in_epoch = h->prog.step_in_epoch;
    sh.lr = h->cfg.lr; sh.momentum = h->cfg.momentum; sh.wd = h->cfg.wd; sh.P = P; sh.R = R;
    sh.optimizer = (uint32_t)h->cfg.optimizer;
    if (h->adam()) { sh.beta2 = h->cfg.beta2; sh.eps = h->cfg.eps; }
    memcpy(hdr, &sh, sizeof(sh));
    char* dst = (char*)dev_dst;
    HIP_TRY(hipMemcpyAsync(dst, hdr, sizeof(hdr), hipMemcpyHostToDevice, h->st));
    HIP_TRY(hipStreamSynchronize(h->st));   // hdr is on this stack frame
    launch_copy(dst + EDL_SNAPSHOT_HEADER_BYTES, h->w(), 4 * (size_t)P, h->st);
    launch_copy(dst + EDL_SNAPSHOT_HEADER_BYTES + 4 * (size_t)P, h->v(), 4 * (size_t)P, h->st);
    size_t at = EDL_SNAPSHOT_HEADER_BYTES + 8 * (size_t)P;
    if (h->adam()) { launch_copy(dst + at, h->s2(), 4 * (size_t)P, h->st); at += 4 * (size_t)P; }
    launch_copy(dst + at, h->running(), 4 * (size_t)R, h->st);
    HIP_TRY(hipGetLastError());
    if (out_written) *out_written = need;
    return EDL_OK;
}

int32_t edl_restore(edl_handle* h, const void* dev_src, size_t len) {
    if (!h || !dev_src) { set_error("null argument"); return EDL_EINVAL; }
    const int64_t P = h->g.P, R = h->g.R;
    const size_t need = EDL_SNAPSHOT_HEADER_BYTES + 4 * (size_t)h->state_floats();
    if (len < need) { set_error("snapshot image of %zu bytes is shorter than %zu", len, need); return EDL_ERANGE; }
    SnapshotHeader sh;
    HIP_TRY(hipMemcpyAsync(&sh, dev_src, sizeof(sh), hipMemcpyDeviceToHost, h->st));
    HIP_TRY(hipStreamSynchronize(h->st));
    if (sh.magic != EDL_SNAPSHOT_MAGIC || sh.version != 1) { set_error("not a snapshot image"); return EDL_EINVAL; }
    if (sh.P != P || sh.R != R || (int32_t)sh.model != h->cfg.model) { set_error("snapshot is of another model (P=%lld, R=%lld)", (long long)sh.P, (long long)sh.R); return EDL_EINVAL; }
    if (sh.N != h->cfg.N || sh.B != h->cfg.B) { set_error("snapshot is of a job with N=%lld B=%lld", (long long)sh.N, (long long)sh.B); return EDL_EINVAL; }
    if ((int32_t)sh.optimizer != h->cfg.optimizer) { set_error("snapshot is of a job with optimizer %u", sh.optimizer); return EDL_EINVAL; }
    if ((int32_t)sh.dtype != h->cfg.dtype) { set_error("snapshot is of a job with dtype %u, this worker was created for %d", sh.dtype, h->cfg.dtype); return EDL_EINVAL; }
    if (!std::isfinite(sh.lr) || !std::isfinite(sh.momentum) || !std::isfinite(sh.wd)) { set_error("snapshot header holds non-finite hyper-parameters"); return EDL_EINVAL; }
    if (h->adam() && !(sh.momentum >= 0.f && sh.momentum < 1.f && sh.beta2 >= 0.f && sh.beta2 < 1.f && sh.eps >= 0.f)) {
        set_error("snapshot header holds Adam coefficients outside their range");
        return EDL_EINVAL;
    }
    const char* src = (const char*)dev_src;
    launch_copy(h->w(), src + EDL_SNAPSHOT_HEADER_BYTES, 4 * (size_t)P, h->st);
    launch_copy(h->v(), src + EDL_SNAPSHOT_HEADER_BYTES + 4 * (size_t)P, 4 * (size_t)P, h->st);
    size_t at = EDL_SNAPSHOT_HEADER_BYTES + 8 * (size_t)P;
    if (h->adam()) { launch_copy(h->s2(), src + at, 4 * (size_t)P, h->st); at += 4 * (size_t)P; }
    launch_copy(h->running(), src + at, 4 * (size_t)R, h->st);
    HIP_TRY(hipGetLastError());
    // job meta-data travels with the model (section 4.2): the joiner takes over the seed, the progress and the
    // optimizer's coefficients, whatever it was created with
    h->seed = sh.seed;
    h->cfg.lr = sh.lr; h->cfg.momentum = sh.momentum; h->cfg.wd = sh.wd;
    if (h->adam()) { h->cfg.beta2 = sh.beta2; h->cfg.eps = sh.eps; }
    h->grads_pending = false;               // gradients of the model that was replaced are void
    h->prog.step = sh.step; h->prog.epoch = sh.epoch; h->prog.step_in_epoch = sh.step_in_epoch;
    h->perm_epoch = -1;
    h->weights_dirty = true;
    return EDL_OK;
}

int32_t edl_get_progress(const edl_handle* h, edl_progress* out) {
    if (!h || !out) { set_error("null argument"); return EDL_EINVAL; }
    *out = h->prog;
    return EDL_OK;
}

static int d2h(edl_handle* h, float* dst, const float* src, int64_t n) {
    if (!h || !dst) { set_error("null argument"); return EDL_EINVAL; }
    HIP_TRY(hipMemcpyAsync(dst, src, sizeof(float) * (size_t)n, hipMemcpyDeviceToHost, h->st));
    HIP_TRY(hipStreamSynchronize(h->st));
    return EDL_OK;
}

int32_t edl_get_params(edl_handle* h, float* host_dst) { return h ? d2h(h, host_dst, h->w(), h->g.P) : EDL_EINVAL; }
int32_t edl_get_momentum(edl_handle* h, float* host_dst) { return h ? d2h(h, host_dst, h->v(), h->g.P) : EDL_EINVAL; }
int32_t edl_get_second_moment(edl_handle* h, float* host_dst) {
    if (!h || !h->adam()) { set_error("not an Adam job"); return EDL_EINVAL; }
    return d2h(h, host_dst, h->s2(), h->g.P);
}
int32_t edl_get_running(edl_handle* h, float* host_dst) { return h ? d2h(h, host_dst, h->running(), h->g.R) : EDL_EINVAL; }
int32_t edl_get_grad(edl_handle* h, int32_t k, float* host_dst) {
    if (!h || k < 0 || k >= h->cfg.p_max) { set_error("gradient buffer %d outside [0,p_max)", k); return EDL_EINVAL; }
    return d2h(h, host_dst, h->grad_buf(k), h->g.P);
}
int32_t edl_get_losses(edl_handle* h, int32_t p, float* host_dst) {
    if (!h || p <= 0 || p > kMaxP) { set_error("bad p"); return EDL_EINVAL; }
    return d2h(h, host_dst, h->at<float>(h->L.losses), p);
}

int32_t edl_set_params(edl_handle* h, const float* host_src) {
    if (!h || !host_src) { set_error("null argument"); return EDL_EINVAL; }
    HIP_TRY(hipMemcpyAsync(h->w(), host_src, sizeof(float) * (size_t)h->g.P, hipMemcpyHostToDevice, h->st));
    HIP_TRY(hipStreamSynchronize(h->st));
    h->weights_dirty = true;
    return EDL_OK;
}

// ---------------------------------------------------------------- debugging hooks
static inline float host_bf16_to_f32(uint16_t v) { uint32_t u = (uint32_t)v << 16; float f; memcpy(&f, &u, 4); return f; }
static inline uint16_t host_f32_to_bf16(float f) {
    uint32_t u; memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

int32_t edl_debug_tensor_count(const edl_handle* h, int32_t* out) {
    if (!h || !out) { set_error("null argument"); return EDL_EINVAL; }
    *out = (int32_t)h->g.tensors.size();
    return EDL_OK;
}

int32_t edl_debug_tensor_shape(const edl_handle* h, int32_t t, int32_t* H, int32_t* W, int32_t* C, int32_t* alias_of) {
    if (!h || t < 0 || (size_t)t >= h->g.tensors.size()) { set_error("tensor %d out of range", t); return EDL_ERANGE; }
    const Tensor& x = h->g.tensors[(size_t)t];
    if (H) *H = x.H;
    if (W) *W = x.W;
    if (C) *C = x.C;
    if (alias_of) *alias_of = x.alias_of;
    return EDL_OK;
}

static int debug_prepare(edl_handle* h, int32_t n) {
    if (!h) { set_error("null handle"); return EDL_EINVAL; }
    if (n <= 0 || n > h->cfg.max_shard || n > h->cfg.B) { set_error("n=%d outside [1, max_shard]", n); return EDL_EINVAL; }
    if (h->weights_dirty) { refresh_weight_copies(h); h->weights_dirty = false; }
    transpose_weights(h, h->st);
    return EDL_OK;
}

int32_t edl_debug_forward(edl_handle* h, const int64_t* idx, int32_t n) {
    int rc = debug_prepare(h, n);
    if (rc) return rc;
    if (!idx || !h->data_x) { set_error("idx and a bound data set are needed"); return EDL_EINVAL; }
    for (int i = 0; i < n; ++i)
        if (idx[i] < 0 || idx[i] >= h->cfg.N) { set_error("idx[%d] outside [0,N)", i); return EDL_ERANGE; }
    HIP_TRY(hipStreamSynchronize(h->st));
    memcpy(h->idx_host[0], idx, sizeof(int64_t) * (size_t)n);
    HIP_TRY(hipMemcpyAsync(h->at<int64_t>(h->L.idx), h->idx_host[0], sizeof(int64_t) * (size_t)n, hipMemcpyHostToDevice, h->st));
    forward_shard(h, h->at<int64_t>(h->L.idx), n, h->at<float>(h->L.losses), false);
    HIP_TRY(hipStreamSynchronize(h->st));
    HIP_TRY(hipGetLastError());
    return EDL_OK;
}

int32_t edl_debug_backward(edl_handle* h, int32_t n, int32_t k) {
    int rc = debug_prepare(h, n);
    if (rc) return rc;
    if (k < 0 || k >= h->cfg.p_max) { set_error("gradient buffer %d outside [0,p_max)", k); return EDL_EINVAL; }
    const Graph& g = h->g;
    launch_softmax_ce(h->cfg.dtype, (const float*)h->act(g.logits), h->at<int32_t>(h->L.labels), h->grad(g.logits),
                      h->sc<float>(h->L.row_loss), h->at<float>(h->L.losses), n, g.classes, h->st);
    backward_shard(h, n, h->grad_buf(k));
    HIP_TRY(hipStreamSynchronize(h->st));
    HIP_TRY(hipGetLastError());
    return EDL_OK;
}

int32_t edl_debug_op_count(const edl_handle* h, int32_t* out) {
    if (!h || !out) { set_error("null argument"); return EDL_EINVAL; }
    *out = (int32_t)h->g.ops.size();
    return EDL_OK;
}

int32_t edl_debug_forward_op(edl_handle* h, int32_t op, int32_t n) {
    int rc = debug_prepare(h, n);
    if (rc) return rc;
    if (op < 0 || (size_t)op >= h->g.ops.size()) { set_error("layer %d out of range", op); return EDL_ERANGE; }
    forward_shard(h, nullptr, n, h->at<float>(h->L.losses), false, (size_t)op, (size_t)op + 1);
    HIP_TRY(hipStreamSynchronize(h->st));
    HIP_TRY(hipGetLastError());
    return EDL_OK;
}

int32_t edl_debug_forward_range(edl_handle* h, int32_t op_lo, int32_t op_hi, int32_t n) {
    int rc = debug_prepare(h, n);
    if (rc) return rc;
    if (op_lo < 0 || op_hi < op_lo || (size_t)op_hi > h->g.ops.size()) { set_error("layers [%d, %d) out of range", op_lo, op_hi); return EDL_ERANGE; }
    forward_shard(h, nullptr, n, h->at<float>(h->L.losses), false, (size_t)op_lo, (size_t)op_hi);
    HIP_TRY(hipStreamSynchronize(h->st));
    HIP_TRY(hipGetLastError());
    return EDL_OK;
}

int32_t edl_debug_backward_op(edl_handle* h, int32_t op, int32_t n, int32_t k) {
    int rc = debug_prepare(h, n);
    if (rc) return rc;
    if (op < 0 || (size_t)op >= h->g.ops.size()) { set_error("layer %d out of range", op); return EDL_ERANGE; }
    if (k < 0 || k >= h->cfg.p_max) { set_error("gradient buffer %d outside [0,p_max)", k); return EDL_EINVAL; }
    backward_shard(h, n, h->grad_buf(k), (size_t)op, (size_t)op + 1);
    HIP_TRY(hipStreamSynchronize(h->st));
    HIP_TRY(hipGetLastError());
    return EDL_OK;
}

int32_t edl_debug_backward_range(edl_handle* h, int32_t op_lo, int32_t op_hi, int32_t n, int32_t k) {
    return edl_debug_backward_range_from(h, op_lo, op_hi, n, k, nullptr, 0);
}

int32_t edl_debug_backward_range_from(edl_handle* h, int32_t op_lo, int32_t op_hi, int32_t n, int32_t k,
                                      const int32_t* held, int32_t n_held) {
    int rc = debug_prepare(h, n);
    if (rc) return rc;
    if (op_lo < 0 || op_hi < op_lo || (size_t)op_hi > h->g.ops.size()) { set_error("layers [%d, %d) out of range", op_lo, op_hi); return EDL_ERANGE; }
    if (k < 0 || k >= h->cfg.p_max) { set_error("gradient buffer %d outside [0,p_max)", k); return EDL_EINVAL; }
    if (n_held < 0 || (n_held > 0 && !held)) { set_error("bad list of held tensors"); return EDL_EINVAL; }
    std::vector<int> hv;
    for (int32_t i = 0; i < n_held; ++i) {
        if (held[i] <= 0 || (size_t)held[i] >= h->g.tensors.size()) { set_error("held tensor %d out of range", held[i]); return EDL_ERANGE; }
        hv.push_back(held[i]);
    }
    backward_shard(h, n, h->grad_buf(k), (size_t)op_lo, (size_t)op_hi, 0, &hv);
    HIP_TRY(hipStreamSynchronize(h->st));
    HIP_TRY(hipGetLastError());
    return EDL_OK;
}


int32_t edl_debug_set_labels(edl_handle* h, const int32_t* labels, int32_t n) {
    if (!h || !labels || n <= 0 || n > h->cfg.max_shard) { set_error("bad argument"); return EDL_EINVAL; }
    HIP_TRY(hipMemcpyAsync(h->at<int32_t>(h->L.labels), labels, sizeof(int32_t) * (size_t)n, hipMemcpyHostToDevice, h->st));
    HIP_TRY(hipStreamSynchronize(h->st));
    return EDL_OK;
}

static int debug_tensor_ptr(edl_handle* h, int32_t t, int32_t which, int32_t n, char** ptr, int64_t* elems, bool* is_f32) {
    if (!h) { set_error("null handle"); return EDL_EINVAL; }
    if (t < 0 || (size_t)t >= h->g.tensors.size()) { set_error("tensor %d out of range", t); return EDL_ERANGE; }
    if (n <= 0 || n > h->cfg.max_shard) { set_error("n=%d outside [1, max_shard]", n); return EDL_EINVAL; }
    const int s = storage_of(h->g, t);
    if (which == 1 && s == 0) { set_error("the input image has no gradient buffer"); return EDL_EINVAL; }
    *ptr = which == 0 ? (char*)h->act(t) : (char*)h->grad(t);
    *elems = h->g.tensors[(size_t)t].elems() * n;
    if (s == 0 && h->L.cpad != h->g.tensors[0].C) { set_error("the input batch is stored channel-padded; it is set by edl_debug_forward only"); return EDL_EINVAL; }
    *is_f32 = h->cfg.dtype == EDL_DTYPE_F32 || (which == 0 && h->g.tensors[(size_t)s].fp32);
    return EDL_OK;
}

int32_t edl_debug_get_tensor(edl_handle* h, int32_t t, int32_t which, int32_t n, float* host_dst) {
    char* ptr; int64_t elems; bool f32;
    const int rc = debug_tensor_ptr(h, t, which, n, &ptr, &elems, &f32);
    if (rc) return rc;
    if (!host_dst) { set_error("null argument"); return EDL_EINVAL; }
    if (f32) {
        HIP_TRY(hipMemcpyAsync(host_dst, ptr, 4 * (size_t)elems, hipMemcpyDeviceToHost, h->st));
        HIP_TRY(hipStreamSynchronize(h->st));
    } else {
        std::vector<uint16_t> tmp((size_t)elems);
        HIP_TRY(hipMemcpyAsync(tmp.data(), ptr, 2 * (size_t)elems, hipMemcpyDeviceToHost, h->st));
        HIP_TRY(hipStreamSynchronize(h->st));
        for (int64_t i = 0; i < elems; ++i) host_dst[i] = host_bf16_to_f32(tmp[(size_t)i]);
    }
    return EDL_OK;
}

int32_t edl_debug_set_tensor(edl_handle* h, int32_t t, int32_t which, int32_t n, const float* host_src) {
    char* ptr; int64_t elems; bool f32;
    const int rc = debug_tensor_ptr(h, t, which, n, &ptr, &elems, &f32);
    if (rc) return rc;
    if (!host_src) { set_error("null argument"); return EDL_EINVAL; }
    if (f32) {
        HIP_TRY(hipMemcpyAsync(ptr, host_src, 4 * (size_t)elems, hipMemcpyHostToDevice, h->st));
        HIP_TRY(hipStreamSynchronize(h->st));
    } else {
        std::vector<uint16_t> tmp((size_t)elems);
        for (int64_t i = 0; i < elems; ++i) tmp[(size_t)i] = host_f32_to_bf16(host_src[i]);
        HIP_TRY(hipMemcpyAsync(ptr, tmp.data(), 2 * (size_t)elems, hipMemcpyHostToDevice, h->st));
        HIP_TRY(hipStreamSynchronize(h->st));
    }
    return EDL_OK;
}

int32_t edl_set_momentum(edl_handle* h, const float* host_src) {
    if (!h || !host_src) { set_error("null argument"); return EDL_EINVAL; }
    HIP_TRY(hipMemcpyAsync(h->v(), host_src, sizeof(float) * (size_t)h->g.P, hipMemcpyHostToDevice, h->st));
    HIP_TRY(hipStreamSynchronize(h->st));
    return EDL_OK;
}

int32_t edl_set_second_moment(edl_handle* h, const float* host_src) {
    if (!h || !host_src) { set_error("null argument"); return EDL_EINVAL; }
    if (!h->adam()) { set_error("not an Adam job"); return EDL_EINVAL; }
    HIP_TRY(hipMemcpyAsync(h->s2(), host_src, sizeof(float) * (size_t)h->g.P, hipMemcpyHostToDevice, h->st));
    HIP_TRY(hipStreamSynchronize(h->st));
    return EDL_OK;
}

int32_t edl_shutdown(edl_handle* h) {
    if (!h) { set_error("null handle"); return EDL_EINVAL; }
    destroy_handle(h);
    return EDL_OK;
}

int32_t edl_profile(int32_t enable) {
    prof_enable(enable != 0);
    return EDL_OK;
}

int32_t edl_profile_report(char* buf, size_t cap, size_t* out_needed) {
    const long n = prof_report(buf, cap);
    if (n < 0) { set_error("reading the timing events failed"); return EDL_EHIP; }
    if (out_needed) *out_needed = (size_t)n + 1;
    if ((size_t)n + 1 > cap) { set_error("report needs %ld bytes", n + 1); return EDL_ENOMEM; }
    return EDL_OK;
}

int32_t edl_average_update(int32_t p, const float* const* dev_grads, float* dev_w, float* dev_v, uint16_t* dev_w16,
                           int64_t P, float lr, float momentum, float wd, void* hip_stream) {
    if (!dev_grads || !dev_w || !dev_v) { set_error("null argument"); return EDL_EINVAL; }
    if (p <= 0 || p > kMaxP) { set_error("p=%d outside [1,%d]", p, kMaxP); return EDL_EINVAL; }
    if (P < 0) { set_error("negative P"); return EDL_EINVAL; }
    if (P == 0) return EDL_OK;
    GradPtrs gp = {};
    uintptr_t bits = (uintptr_t)dev_w | (uintptr_t)dev_v | (uintptr_t)dev_w16;
    for (int k = 0; k < p; ++k) {
        if (!dev_grads[k]) { set_error("gradient pointer %d is NULL", k); return EDL_EINVAL; }
        gp.g[k] = dev_grads[k];
        bits |= (uintptr_t)dev_grads[k];
    }
    if (bits & 15) { set_error("pointers must be 16-byte aligned"); return EDL_EINVAL; }
    launch_average_update(p, gp, dev_w, dev_v, dev_w16, P, lr, momentum, wd, (hipStream_t)hip_stream);
    HIP_TRY(hipGetLastError());
    return EDL_OK;
}

int32_t edl_adam_update(int32_t p, const float* const* dev_grads, const float* shares, float* dev_w, float* dev_m,
                        float* dev_s, uint16_t* dev_w16, int64_t P, float lr, float beta1, float beta2, float eps,
                        float wd, int64_t t, void* hip_stream) {
    if (!dev_grads || !dev_w || !dev_m || !dev_s) { set_error("null argument"); return EDL_EINVAL; }
    if (p <= 0 || p > kMaxP) { set_error("p=%d outside [1,%d]", p, kMaxP); return EDL_EINVAL; }
    if (P < 0 || t < 1) { set_error("negative P or t < 1"); return EDL_EINVAL; }
    if (!(beta1 >= 0.f && beta1 < 1.f && beta2 >= 0.f && beta2 < 1.f && eps >= 0.f)) { set_error("betas must lie in [0,1), eps >= 0"); return EDL_EINVAL; }
    if (P == 0) return EDL_OK;
    GradPtrs gp = {};
    ShardShares sh = {};
    uintptr_t bits = (uintptr_t)dev_w | (uintptr_t)dev_m | (uintptr_t)dev_s | (uintptr_t)dev_w16;
    for (int k = 0; k < p; ++k) {
        if (!dev_grads[k]) { set_error("gradient pointer %d is NULL", k); return EDL_EINVAL; }
        gp.g[k] = dev_grads[k];
        bits |= (uintptr_t)dev_grads[k];
        if (shares) sh.share[k] = shares[k];
    }
    if (bits & 15) { set_error("pointers must be 16-byte aligned"); return EDL_EINVAL; }
    float c1, c2;
    adam_corrections(beta1, beta2, t, &c1, &c2);
    launch_adam_update(p, gp, shares ? &sh : nullptr, dev_w, dev_m, dev_s, dev_w16, P, lr, beta1, beta2, eps, wd, c1, c2,
                       (hipStream_t)hip_stream);
    HIP_TRY(hipGetLastError());
    return EDL_OK;
}

int32_t edl_mfma_rate(int32_t dtype, int32_t blocks, int32_t iters, float* dev_sink, void* hip_stream, double* out_flops) {
    if ((dtype != EDL_DTYPE_F32 && dtype != EDL_DTYPE_BF16) || blocks <= 0 || blocks > (1 << 20) || iters <= 0 || !dev_sink) {
        set_error("bad argument");
        return EDL_EINVAL;
    }
    const double flops = launch_mfma_rate(dtype, blocks, iters, dev_sink, (hipStream_t)hip_stream);
    if (out_flops) *out_flops = flops;
    HIP_TRY(hipGetLastError());
    return EDL_OK;
}

int32_t edl_copy(void* dev_dst, const void* dev_src, size_t bytes, void* hip_stream) {
    if (!dev_dst || !dev_src) { set_error("null argument"); return EDL_EINVAL; }
    launch_copy(dev_dst, dev_src, bytes, (hipStream_t)hip_stream);
    HIP_TRY(hipGetLastError());
    return EDL_OK;
}

}  // extern "C"
