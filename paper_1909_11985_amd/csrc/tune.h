// Behaviour switches and launch heuristics of the library, in one table.
// Every entry starts at its measured-best default, can be preset from the
// environment (EDL_TUNE_<NAME in capitals>, read once when the table is first
// used) and changed at run time through edl_set_option(name, value).  The
// launchers read plain fields, so a changed value holds from the next launch
// on; values only choose between code paths that give the same results up to
// summation order (tile shapes, reduction cuts, streams), never what is
// computed.  Host only.
#pragma once
#include <cstdint>

namespace edl {

struct Tune {
    int64_t min128 = 256;             // tiles a forward / dgrad problem needs before the 128x128 tile is chosen
    int64_t min128_long = 160;        // ... when its reduction has 4,096 or more elements
    int64_t force_tile = -1;          // 0..3: every forward / dgrad launch on 128x128, 128x64, 128x32, 64x64 tiles
    int64_t bk64_kred = 1024;         // 128x128 tiles take full-length reduction steps from this reduction length on
    int64_t xcd = 1;                  // die-chunked tile order
    int64_t order = -1;               // -1: tile order by operand size; 0 / 1: rows / columns fastest
    int64_t splitk_tiles = 300;       // forward / dgrad problems of fewer tiles have their reduction cut ...
    int64_t splitk_target = 320;      // ... towards this many workgroups
    int64_t fused_stats = 1;          // batch-norm sums out of the forward convolution's epilogue
    int64_t held_stats = 1;           // ... also for a block's last convolution, held while the shortcut's batch norm runs
    int64_t fused_mask = 1;           // masked gradient + backward sums out of the dgrad epilogue
    int64_t fused_mask_cut = 1;       // ... out of the finishing kernel where the dgrad's reduction is cut
    int64_t fused_mask_join = 1;      // ... at a residual join (the epilogue adds to the shortcut's part first)
    int64_t join_tile = 1;            // 128x64 tiles for the join epilogue
    int64_t small_tail_from = 768;    // 64x64 forward / dgrad launches of more workgroups than this (three per CU) ...
    int64_t small_tail_to = 1280;     // ... and at most this many (five per CU) run the two-stage form, all workgroups resident at once
    int64_t wgrad_blocks = 128;       // workgroups a weight gradient is cut towards
    int64_t wgrad_long_blocks = 512;  // ... for long reductions
    int64_t wgrad_long_ks = 3072;     // least reduction elements per cut of a long reduction
    int64_t wgrad_deep_max = 256;     // weight gradients of at most this many workgroups keep one more tile in flight (0: none do)
    int64_t wgrad_stream = 1;         // weight gradients on a second stream (read when a job is created)
    int64_t wgrad_tail_main = 1;      // the first this-many convolutions keep their weight gradient on the main stream
    int64_t early_update = 16000000;  // layers of at least this many weights start their update during the backward pass (0: none)
    int64_t early_blocks = 256;       // workgroups of such a background update
    int64_t upd_vpt = 1;              // 16-byte vectors per lane of the update kernel (1 or 2)
    int64_t upd_wide = -1;            // > 0: the update walks its streams in wave-wide pieces, this many vectors per lane (1, 2, 4); -1: chosen by the launcher (array placement, p); 0: one vector per lane, plain loads
    int64_t upd_nt = -1;              // ... non-temporal accesses: bit 0 gradient loads, bit 1 bf16 store, bit 2 w and v; -1: chosen by the launcher
    int64_t upd_blocks = 0;           // ... > 0: grid-stride launch of this many workgroups
    int64_t branch_stream = 1;        // a residual block's projection shortcut runs on the second side stream beside the main branch
    int64_t transpose_stream = 0;     // 1: the transposed weight copies are made on the weight-gradient stream during the forward pass (measured: no gain, 4.499 vs 4.509 ms)
    int64_t alias_shortcut = 1;       // an identity shortcut's gradient is read from the block output's gradient instead of being copied
    int64_t bn_nt = 1;                // the batch-norm element-wise passes load what they read once (the convolution's output; the activation for the mask) non-temporally ...
    int64_t bn_nt_bytes = 8000000;    // ... for tensors of at least this many bytes
    int64_t spare0 = 0, spare1 = 0;   // free slots for experiments (EDL_TUNE_SPARE0 / 1)
};

// The process-wide table (loaded from the environment on first use).
Tune& tune();
// Sets one entry by its field name; returns false if there is no such entry.
bool tune_set(const char* name, int64_t value);
// Reads one entry by name into *value; returns false if there is no such entry.
bool tune_get(const char* name, int64_t* value);

}  // namespace edl
