// Dynamic data pipeline (section 4.3 of the paper): the leader's bookkeeping.
// The data set is cut into d partitions at the meta-data level; a permutation
// of the partitions is drawn per epoch; a worker that needs data is given the
// next piece (a handed-back remainder first, else the next unassigned
// partition) and reads it front to back; a worker that leaves hands the rest
// of its partition back.  Host only, integers only.
#include <algorithm>
#include <cstring>
#include <deque>
#include <new>
#include <vector>

#include "../../include/edl.h"
#include "graph.h"

namespace {

struct Piece {
    int64_t part, pos;          // partition and the sample index its next read starts at
};

struct Holder {
    int64_t id;                 // caller's name of the worker
    Piece piece;                // pos == end of the partition: nothing held
};

constexpr int64_t kImageMagic = 0x45444c50495045ll;   // "EDLPIPE"
constexpr int64_t kImageVersion = 1;

}  // namespace

struct edl_pipeline {
    uint64_t seed = 0;
    int64_t N = 0, d = 0, span = 0;      // span = samples per partition (the last one may be shorter)
    int64_t epoch = 0, consumed = 0, cursor = 0;
    std::vector<int64_t> order;          // this epoch's permutation of the partitions
    std::deque<Piece> returned;          // handed-back remainders, first in first out
    std::vector<Holder> holders;         // what each known worker holds
    std::vector<int64_t> ranks;          // the previous mini-batch's workers in rank order

    int64_t part_end(int64_t part) const { return std::min((part + 1) * span, N); }

    Holder* find(int64_t id) {
        for (Holder& h : holders)
            if (h.id == id) return &h;
        return nullptr;
    }

    void start_epoch(int64_t e) {
        epoch = e;
        consumed = 0;
        cursor = 0;
        returned.clear();
        holders.clear();
        edl::epoch_permutation(seed, e, d, order);
    }

    // the next piece the leader hands out; false if the epoch has none left
    bool hand_out(Piece* out) {
        if (!returned.empty()) {
            *out = returned.front();
            returned.pop_front();
            return true;
        }
        if (cursor < d) {
            const int64_t part = order[(size_t)cursor++];
            *out = Piece{part, part * span};
            return true;
        }
        return false;
    }

    // up to `want` samples for worker `id`, written from dst on; returns how many
    int64_t draw(int64_t id, int64_t want, int64_t* dst) {
        int64_t got = 0;
        while (got < want) {
            Holder* h = find(id);
            if (!h || h->piece.pos >= part_end(h->piece.part)) {
                Piece fresh;
                if (!hand_out(&fresh)) break;
                if (!h) {
                    holders.push_back(Holder{id, fresh});
                    h = &holders.back();
                } else {
                    h->piece = fresh;
                }
            }
            const int64_t take = std::min(want - got, part_end(h->piece.part) - h->piece.pos);
            for (int64_t i = 0; i < take; ++i) dst[got + i] = h->piece.pos + i;
            h->piece.pos += take;
            got += take;
        }
        return got;
    }
};

extern "C" {

int32_t edl_pipeline_create(uint64_t seed, int64_t N, int64_t d, edl_pipeline** out) {
    if (!out) { edl::set_error("null argument"); return EDL_EINVAL; }
    *out = nullptr;
    if (N <= 0 || d <= 0 || d > N) { edl::set_error("need 0 < d <= N (d=%lld, N=%lld)", (long long)d, (long long)N); return EDL_EINVAL; }
    const int64_t span = (N + d - 1) / d;
    if ((d - 1) * span >= N) {
        edl::set_error("%lld partitions of %lld samples leave a partition empty", (long long)d, (long long)span);
        return EDL_EINVAL;
    }
    edl_pipeline* p = new (std::nothrow) edl_pipeline();
    if (!p) { edl::set_error("out of host memory"); return EDL_ENOMEM; }
    p->seed = seed; p->N = N; p->d = d; p->span = span;
    p->start_epoch(0);
    *out = p;
    return EDL_OK;
}

int32_t edl_pipeline_next_batch(edl_pipeline* pl, int64_t B, int32_t p, const int64_t* worker_ids, int64_t* out_idx,
                                int64_t* out_off) {
    if (!pl || !worker_ids || !out_idx || !out_off) { edl::set_error("null argument"); return EDL_EINVAL; }
    if (p <= 0 || B <= 0) { edl::set_error("p and B must be positive"); return EDL_EINVAL; }
    if (B % p || pl->N % B) { edl::set_error("B=%lld must divide N=%lld and be a multiple of p=%d", (long long)B, (long long)pl->N, p); return EDL_EINDIVISIBLE; }
    for (int a = 0; a < p; ++a)
        for (int b = a + 1; b < p; ++b)
            if (worker_ids[a] == worker_ids[b]) { edl::set_error("worker id %lld appears twice", (long long)worker_ids[a]); return EDL_EINVAL; }
    if (pl->consumed == pl->N) pl->start_epoch(pl->epoch + 1);
    // graceful exits: whoever was in the previous mini-batch and is not in this one hands back, in old rank order
    for (int64_t old : pl->ranks) {
        if (std::find(worker_ids, worker_ids + p, old) != worker_ids + p) continue;
        for (size_t i = 0; i < pl->holders.size(); ++i) {
            if (pl->holders[i].id != old) continue;
            const Piece pc = pl->holders[i].piece;
            if (pc.pos < pl->part_end(pc.part)) pl->returned.push_back(pc);
            pl->holders.erase(pl->holders.begin() + (long)i);
            break;
        }
    }
    pl->ranks.assign(worker_ids, worker_ids + p);
    // Rank order, B/p samples each; what a worker cannot be given is passed on to the next ones.  A worker
    // asked twice (second round) appends to its own shard, so the shards are gathered per worker first.
    const int64_t n = B / p;
    std::vector<std::vector<int64_t>> shard((size_t)p);
    std::vector<int64_t> tmp((size_t)B);
    int64_t lacking = 0;
    for (int k = 0; k < p; ++k) {
        const int64_t want = n + lacking;
        const int64_t got = pl->draw(worker_ids[k], want, tmp.data());
        shard[(size_t)k].assign(tmp.begin(), tmp.begin() + got);
        lacking = want - got;
    }
    for (int k = 0; k < p && lacking > 0; ++k) {
        const int64_t got = pl->draw(worker_ids[k], lacking, tmp.data());
        shard[(size_t)k].insert(shard[(size_t)k].end(), tmp.begin(), tmp.begin() + got);
        lacking -= got;
    }
    if (lacking > 0) { edl::set_error("the epoch ran out inside a mini-batch"); return EDL_ERANGE; }
    int64_t at = 0;
    out_off[0] = 0;
    for (int k = 0; k < p; ++k) {
        std::copy(shard[(size_t)k].begin(), shard[(size_t)k].end(), out_idx + at);
        at += (int64_t)shard[(size_t)k].size();
        out_off[k + 1] = at;
    }
    pl->consumed += B;
    return EDL_OK;
}

int32_t edl_pipeline_progress(const edl_pipeline* pl, int64_t* out_epoch, int64_t* out_consumed) {
    if (!pl) { edl::set_error("null argument"); return EDL_EINVAL; }
    if (out_epoch) *out_epoch = pl->epoch;
    if (out_consumed) *out_consumed = pl->consumed;
    return EDL_OK;
}

int32_t edl_pipeline_save(const edl_pipeline* pl, int64_t* buf, size_t cap_words, size_t* out_words) {
    if (!pl) { edl::set_error("null argument"); return EDL_EINVAL; }
    const size_t need = 11 + 2 * pl->returned.size() + pl->ranks.size() + 3 * pl->holders.size();
    if (out_words) *out_words = need;
    if (!buf || cap_words < need) { edl::set_error("the image needs %zu words", need); return EDL_ENOMEM; }
    size_t at = 0;
    const int64_t head[11] = {kImageMagic, kImageVersion, (int64_t)pl->seed, pl->N, pl->d, pl->epoch, pl->consumed, pl->cursor,
                              (int64_t)pl->returned.size(), (int64_t)pl->ranks.size(), (int64_t)pl->holders.size()};
    for (int64_t v : head) buf[at++] = v;
    for (const Piece& pc : pl->returned) { buf[at++] = pc.part; buf[at++] = pc.pos; }
    for (int64_t id : pl->ranks) buf[at++] = id;
    for (const Holder& h : pl->holders) { buf[at++] = h.id; buf[at++] = h.piece.part; buf[at++] = h.piece.pos; }
    return EDL_OK;
}

int32_t edl_pipeline_load(const int64_t* buf, size_t words, edl_pipeline** out) {
    if (!buf || !out) { edl::set_error("null argument"); return EDL_EINVAL; }
    *out = nullptr;
    if (words < 11 || buf[0] != kImageMagic || buf[1] != kImageVersion) { edl::set_error("not a pipeline image"); return EDL_EINVAL; }
    const int64_t n_ret = buf[8], n_rank = buf[9], n_hold = buf[10];
    if (n_ret < 0 || n_rank < 0 || n_hold < 0 || (size_t)(11 + 2 * n_ret + n_rank + 3 * n_hold) != words) {
        edl::set_error("pipeline image has the wrong length");
        return EDL_EINVAL;
    }
    edl_pipeline* p = nullptr;
    const int rc = edl_pipeline_create((uint64_t)buf[2], buf[3], buf[4], &p);
    if (rc) return rc;
    const int64_t epoch = buf[5], consumed = buf[6], cursor = buf[7];
    if (epoch < 0 || consumed < 0 || consumed > p->N || cursor < 0 || cursor > p->d) {
        delete p;
        edl::set_error("pipeline image holds impossible progress");
        return EDL_ERANGE;
    }
    p->start_epoch(epoch);
    p->consumed = consumed;
    p->cursor = cursor;
    size_t at = 11;
    auto piece_ok = [&](const Piece& pc) { return pc.part >= 0 && pc.part < p->d && pc.pos >= pc.part * p->span && pc.pos <= p->part_end(pc.part); };
    bool ok = true;
    for (int64_t i = 0; i < n_ret; ++i) { const Piece pc{buf[at], buf[at + 1]}; at += 2; ok = ok && piece_ok(pc); p->returned.push_back(pc); }
    for (int64_t i = 0; i < n_rank; ++i) p->ranks.push_back(buf[at++]);
    for (int64_t i = 0; i < n_hold; ++i) { const Holder h{buf[at], Piece{buf[at + 1], buf[at + 2]}}; at += 3; ok = ok && piece_ok(h.piece); p->holders.push_back(h); }
    if (!ok) {
        delete p;
        edl::set_error("pipeline image holds a piece outside its partition");
        return EDL_ERANGE;
    }
    *out = p;
    return EDL_OK;
}

int32_t edl_pipeline_destroy(edl_pipeline* pl) {
    delete pl;
    return EDL_OK;
}

}  // extern "C"
