// Internal declarations shared by the library's translation units (not part
// of the public ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "fdd.h"

namespace fdd {

// MI355X has 256 compute units in 8 XCDs; grid-shape heuristics are sized
// for that chip and do not query the device, so that workspace sizes are a
// pure function of the problem shape.
constexpr int kNumCU = 256;
constexpr int kNumXCD = 8;

// Stacked-row decomposition of the attention problem.  For one KV head the
// query rows of all rollouts, positions and group heads form one list of
// R = N*B*G rows, r = (n*B + b)*G + g, cut into M-tiles of `mtile_rows`.
// The prefix is cut into `splits` pieces along L; piece s of M-tile mt of
// head kh leaves a partial (m, l, o[D]) in the workspace unless splits == 1.
struct AttnPlan {
    int G;            // query heads per KV head
    int R;            // stacked rows per KV head
    int mtile_rows;   // rows per M-tile
    int MT;           // M-tiles per KV head
    int key_tile;     // keys per streamed tile
    int TP;           // prefix tiles = ceil(L / key_tile)
    int splits;       // pieces along L
    size_t ws_o_bytes;   // partial outputs  [Hkv][MT][splits][mtile_rows][D] fp32
    size_t ws_ml_bytes;  // partial (m, l)   [Hkv][MT][splits][mtile_rows][2] fp32
};

bool make_attn_plan(const fdd_attn_params& p, AttnPlan* plan);

hipError_t launch_attn_bf16(const fdd_attn_params& p, const AttnPlan& plan, float scale, hipStream_t s);
hipError_t launch_attn_f32(const fdd_attn_params& p, const AttnPlan& plan, float scale, hipStream_t s);
hipError_t launch_attn_combine(const fdd_attn_params& p, const AttnPlan& plan, float scale, hipStream_t s);

// Vocabulary reduction: each eligible logits row is cut into `vsplits`
// pieces; a piece leaves (max, argmax, sum exp(x - max)) in the workspace.
struct UnmaskPlan {
    int vsplits;
    size_t ws_bytes;  // [N*B][vsplits] x {float max; int32 arg; float sum; int32 pad}
};
bool make_unmask_plan(const fdd_unmask_params& p, UnmaskPlan* plan);
hipError_t launch_unmask(const fdd_unmask_params& p, const UnmaskPlan& plan, hipStream_t s);

hipError_t launch_fork_block(int N, size_t bytes, const void* src, void* dst, hipStream_t s);
hipError_t launch_kv_update(const fdd_kv_update_params& p, hipStream_t s);

}  // namespace fdd
