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
// R = N*B*G rows, r = (n*B + b)*G + g, cut into M-tiles of `mtile_rows`; an
// M-tile index M = kh*MT + mt runs over all KV heads.  The key range of an
// M-tile is processed in one or more segments; segment `seg` of M-tile M
// leaves a partial (m, l, o[D]) in slot M*max_seg + seg of the workspace
// unless it is the M-tile's only segment.
//   fp32 path : `splits` equal pieces per M-tile, one workgroup each.
//   bf16 path : the unit is one key tile of one M-tile (TPU units per M-tile,
//               U in total).  Either every M-tile is cut into `uniform` equal
//               pieces, piece s covering tiles [TPU s / S, TPU (s+1) / S), or
//               (stream-K) workgroup w of W owns the contiguous unit range
//               [unit_begin(w), unit_begin(w+1)), which may cross M-tiles.
struct AttnPlan {
    int G;            // query heads per KV head
    int R;            // stacked rows per KV head
    int mtile_rows;   // rows per M-tile
    int MT;           // M-tiles per KV head
    int key_tile;     // keys per streamed tile
    int TP;           // prefix tiles = ceil(L / key_tile)
    int splits;       // fp32 path: pieces along L
    int TPU;          // bf16 path: units per M-tile = max(TP, 1)
    int W;            // bf16 path: workgroups
    int uniform;      // bf16 path: > 0 when W = Hkv*MT*uniform, i.e. equal pieces per M-tile
    long long U;      // bf16 path: units in total
    int max_seg;      // partial slots per M-tile
    size_t ws_o_bytes;   // partial outputs  [Hkv*MT][max_seg][mtile_rows][D], fp32 (fp32 path) or bf16 (bf16 path)
    size_t ws_ml_bytes;  // partial (m, l)   [Hkv*MT][max_seg][mtile_rows][2] fp32
    size_t ws_vt_bytes;  // bf16 path: V of the full prefix tiles repacked for the P V fragments, or 0
    bool packed;         // bf16 path: the kernel reads repacked V (from the workspace or from the caller)
};

bool make_attn_plan(const fdd_attn_params& p, AttnPlan* plan);

// Records the message fdd_last_error() returns on this thread; returns `code`.
fdd_status set_error(fdd_status code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
// Host-side checks of an unmask call (everything but the workspace); `fn` names the entry point in messages.
fdd_status check_unmask_args(const fdd_unmask_params* p, const char* fn);

// Division by a number fixed per launch, prepared on the host: for 0 <= n < 2^31 and 1 <= d < 2^31,
// n / d = ((n + 1) * mul) >> (32 + shift), where k = 31 + max(1, ceil(log2 d)), shift = k - 32 and mul is the
// largest integer with mul * d < 2^k.  With e = 2^k - mul * d in (0, d] and n = q d + r the product is
// q + ((r + 1) - (n + 1) e / 2^k) / d, and (n + 1) e <= 2^k keeps the bracket in [r, r + 1).
struct FastDiv {
    uint32_t mul, shift;
};
inline FastDiv make_fastdiv(uint32_t d)
{
    if (d == 0) d = 1;   // never used as a divisor then; keeps the host arithmetic defined
    uint32_t s = 1;
    while ((1ull << s) < d) ++s;
    const uint64_t two_k = 1ull << (31 + s);
    FastDiv f;
    f.mul = (uint32_t)((two_k - 1) / d);
    f.shift = s - 1;
    return f;
}
__device__ __forceinline__ int fast_div(int n, const FastDiv& f)
{
    return (int)((uint32_t)(((uint64_t)((uint32_t)n + 1u) * f.mul) >> 32) >> f.shift);
}

// Stream-K ranges: U units over W workgroups, base = U / W, rem = U % W; the
// first `rem` workgroups own base + 1 units, the others base (>= 1).
__host__ __device__ inline int unit_begin(int w, int base, int rem) { return w * base + (w < rem ? w : rem); }
__host__ __device__ inline int wg_of_unit(int u, int base, int rem)
{
    const int cut = rem * (base + 1);
    return u < cut ? u / (base + 1) : rem + (u - cut) / base;
}

// `before_main`, if not null, is recorded on the stream right before the main kernel (after the V pre-pass).
hipError_t launch_attn_bf16(const fdd_attn_params& p, const AttnPlan& plan, float scale, hipStream_t s, hipEvent_t before_main);
hipError_t launch_prefix_pack(const void* prefix_v, int L, int Hkv, int D, void* packed, hipStream_t s);
hipError_t launch_attn_f32(const fdd_attn_params& p, const AttnPlan& plan, float scale, hipStream_t s);
hipError_t launch_attn_combine(const fdd_attn_params& p, const AttnPlan& plan, float scale, hipStream_t s);      // fp32 path
hipError_t launch_attn_merge_bf16(const fdd_attn_params& p, const AttnPlan& plan, float scale, hipStream_t s);   // bf16 path

// Vocabulary reduction: each eligible logits row is cut into `vsplits`
// pieces; a piece leaves (max, argmax, sum exp(x - max)) in the workspace.
struct UnmaskPlan {
    int vsplits;
    size_t ws_bytes;  // [N*B][vsplits] x {float max; int32 arg; float sum; int32 pad}
};
bool make_unmask_plan(const fdd_unmask_params& p, UnmaskPlan* plan);
// `argmax_only`: the plan of the greedy verifier's pass (no sums); the sampled verifier and the unmask step share the other
bool make_vocab_plan(int N, int B, long long V, int dtype, bool argmax_only, UnmaskPlan* plan);
hipError_t launch_unmask(const fdd_unmask_params& p, const UnmaskPlan& plan, hipStream_t s);
hipError_t launch_verify(const fdd_verify_params& p, const UnmaskPlan& plan, hipStream_t s);

hipError_t launch_fork_block(int N, size_t bytes, const void* src, void* dst, hipStream_t s);
hipError_t launch_kv_update(const fdd_kv_update_params& p, hipStream_t s);
hipError_t launch_block_commit(const fdd_commit_params& p, hipStream_t s);
hipError_t launch_traj_mean(int N, int P, const float* traj, float* out, hipStream_t s);

}  // namespace fdd
