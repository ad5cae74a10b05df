// C ABI entry points: host-side validation, planning and launches.
#include <cmath>
#include <cstdint>
#include <cstdarg>
#include <cstdio>

#include "fdd_internal.h"
#include <algorithm>

namespace fdd {
namespace {

thread_local char g_err[384] = "";
thread_local hipEvent_t g_ev_start = nullptr;
thread_local hipEvent_t g_ev_stop = nullptr;

}  // namespace

fdd_status set_error(fdd_status code, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

namespace {

#define fail set_error

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

fdd_status check_attn_shape(const fdd_attn_params* p)
{
    if (!p) return fail(FDD_ERR_NULL, "fdd_block_attn: params is NULL");
    if (p->N <= 0 || p->B <= 0 || p->L < 0 || p->Hq <= 0 || p->Hkv <= 0 || p->D <= 0)
        return fail(FDD_ERR_SHAPE, "fdd_block_attn: N, B, Hq, Hkv, D must be positive and L >= 0 (got N=%d B=%d L=%d Hq=%d Hkv=%d D=%d)",
                    p->N, p->B, p->L, p->Hq, p->Hkv, p->D);
    if (p->Hq % p->Hkv) return fail(FDD_ERR_SHAPE, "fdd_block_attn: Hq=%d is not a multiple of Hkv=%d", p->Hq, p->Hkv);
    if (p->dtype != FDD_F32 && p->dtype != FDD_BF16) return fail(FDD_ERR_DTYPE, "fdd_block_attn: dtype %d is neither FDD_F32 nor FDD_BF16", p->dtype);
    if (p->D != 64 && p->D != 128) return fail(FDD_ERR_UNSUPPORTED, "fdd_block_attn: head size D=%d not supported (64 or 128)", p->D);
    if (p->splits < 0 || p->splits > 64) return fail(FDD_ERR_UNSUPPORTED, "fdd_block_attn: splits=%d outside [0, 64]", p->splits);
    if (p->flags & ~FDD_ATTN_CAUSAL_BLOCK) return fail(FDD_ERR_UNSUPPORTED, "fdd_block_attn: unknown bits in flags (0x%x)", p->flags);
    // (every product below is bounded before the next factor is multiplied in: no 64-bit overflow for any int32 input)
    const long long nb = (long long)p->N * p->B;
    if (nb > (1ll << 30) || nb * (p->Hq / p->Hkv) > (1ll << 30) || nb * p->Hq > (1ll << 33))
        return fail(FDD_ERR_SHAPE, "fdd_block_attn: N*B*Hq too large");
    if ((long long)p->L * p->Hkv >= (1ll << 31) || (long long)p->L * p->Hkv * p->D * 4 >= (1ll << 31))
        return fail(FDD_ERR_SHAPE, "fdd_block_attn: prefix K (L*Hkv*D elements) must stay below 2 GiB");
    if (nb * p->Hkv >= (1ll << 32) || nb * p->Hkv * p->D * 4 >= (1ll << 32))
        return fail(FDD_ERR_SHAPE, "fdd_block_attn: block K (N*B*Hkv*D elements) must stay below 4 GiB");
    if (p->batch < 0 || p->batch > 65535 / p->Hkv) return fail(FDD_ERR_SHAPE, "fdd_block_attn: batch=%d outside [0, 65535 / Hkv]", p->batch);
    {
        // work units of the bf16 path: (KV head, 256-row M-tile, 64-key prefix tile)
        const long long mt = (nb * (p->Hq / p->Hkv) + 255) / 256;            // <= 2^22
        const long long tpu = (p->L + 63) / 64 + 64;          // prefix tiles plus the units booked for private tiles (bounded by 64 here)
        const long long heads = (long long)p->Hkv * (p->batch > 1 ? p->batch : 1);                 // <= 2^16
        if (heads * mt >= (1ll << 31) || heads * mt * tpu >= (1ll << 31)) return fail(FDD_ERR_SHAPE, "fdd_block_attn: batch*N*B*Hq*L too large");
    }
    if (std::isnan(p->scale) || std::isinf(p->scale)) return fail(FDD_ERR_UNSUPPORTED, "fdd_block_attn: scale is not finite");
    if (p->n_q_positions < 0 || (long long)p->n_q_positions > (long long)p->N * p->B)
        return fail(FDD_ERR_SHAPE, "fdd_block_attn: n_q_positions=%d outside [0, N*B]", p->n_q_positions);
    if (p->batch > 1) {
        const long long es = p->dtype == FDD_BF16 ? 2 : 4;
        struct { const char* name; long long stride, need; } st[] = {
            {"q_batch_stride", p->q_batch_stride, (long long)p->N * p->B * p->Hq * p->D},
            {"out_batch_stride", p->out_batch_stride, (long long)p->N * p->B * p->Hq * p->D},
            {"block_batch_stride", p->block_batch_stride, (long long)p->N * p->B * p->Hkv * p->D},
            {"prefix_batch_stride", p->prefix_batch_stride, (long long)p->L * p->Hkv * p->D},
            {"ext_batch_stride", p->ext_batch_stride, p->E > 0 ? (long long)p->N * p->ext_capacity * p->Hkv * p->D : 0},
        };
        for (const auto& x : st)
            if (x.stride < x.need || (x.stride * es) % 16)
                return fail(FDD_ERR_SHAPE, "fdd_block_attn: %s=%lld must be at least %lld elements and a multiple of 16 bytes",
                            x.name, x.stride, x.need);
        if (p->prefix_v_packed && (p->packed_batch_stride % 256 ||
                                   p->packed_batch_stride < (size_t)p->Hkv * (p->L / 64) * 64 * p->D * 2))
            return fail(FDD_ERR_SHAPE, "fdd_block_attn: packed_batch_stride must be a multiple of 256 and hold one packed prefix V");
    }
    if (p->E < 0 || p->ext_capacity < 0 || p->E > p->ext_capacity)
        return fail(FDD_ERR_SHAPE, "fdd_block_attn: need 0 <= E <= ext_capacity (got E=%d, ext_capacity=%d)", p->E, p->ext_capacity);
    if ((long long)p->N * p->ext_capacity * p->Hkv * p->D * 4 >= (1ll << 32))
        return fail(FDD_ERR_SHAPE, "fdd_block_attn: extension K (N*ext_capacity*Hkv*D elements) must stay below 4 GiB");
    return FDD_OK;
}

}  // namespace

bool make_attn_plan(const fdd_attn_params& p, AttnPlan* plan)
{
    AttnPlan pl;
    pl.G = p.Hq / p.Hkv;
    pl.R = (p.n_q_positions > 0 ? p.n_q_positions : p.N * p.B) * pl.G;
    if (p.dtype == FDD_BF16) {
        pl.mtile_rows = 256;
        pl.key_tile = 64;
    } else {
        pl.mtile_rows = 16;
        pl.key_tile = 32;
    }
    pl.MT = (pl.R + pl.mtile_rows - 1) / pl.mtile_rows;
    pl.TP = (p.L + pl.key_tile - 1) / pl.key_tile;
    const int batch = p.batch > 1 ? p.batch : 1;
    const long long NM = (long long)p.Hkv * batch * pl.MT;
    bool partials;
    if (p.dtype == FDD_BF16) {
        // The private tiles of an M-tile (extension and block of every rollout its rows belong to) are done
        // by the workgroup that ends the M-tile's key range, one after the other and at about 1.8 times the
        // cost of a pipelined prefix tile.  They are booked as `wt` extra units at the end of the M-tile's
        // unit range, so that this workgroup gets correspondingly fewer prefix tiles.
        // (with a list of query positions a rollout contributes fewer rows: its average share stands in for B)
        const long long BG = p.n_q_positions > 0 ? std::max(1ll, (long long)p.n_q_positions * pl.G / p.N) : (long long)p.B * pl.G;
        const long long span_lo = (pl.mtile_rows + BG - 1) / BG;                 // rollouts an M-tile spans at least
        const long long span = span_lo + ((pl.mtile_rows % BG) != 0 && BG < (long long)pl.R ? 1 : 0);
        const long long private_tiles = (span < p.N ? span : p.N) *
                                        ((p.E + pl.key_tile - 1) / pl.key_tile + (p.B + pl.key_tile - 1) / pl.key_tile);
        long long wt = (private_tiles * 9 + 4) / 5;
        if (wt < 1) wt = 1;
        if (wt > 64) wt = 64;
        auto pieces_for = [&](long long tpu) {
            // equal pieces per M-tile, at least two units each; the fewest pieces that reach the shortest critical path
            long long smax = NM > 0 ? kNumCU / NM : 0;
            if (smax > tpu / 2) smax = tpu / 2;
            if (smax < 1) return 0ll;
            const long long crit = (tpu + smax - 1) / smax;
            long long sbest = smax;
            while (sbest > 1 && (tpu + (sbest - 1) - 1) / (sbest - 1) == crit) --sbest;
            return sbest;
        };
        long long w;
        pl.uniform = 0;
        if (p.splits > 0) {
            if (wt > 2) wt = 2;
            pl.TPU = pl.TP + (int)wt;
            pl.uniform = p.splits < pl.TPU ? p.splits : pl.TPU;
            w = NM * pl.uniform;
        } else {
            // Equal pieces per M-tile when that fills at least 4/5 of the compute
            // units: the workgroups of an XCD then walk the same K/V tiles in step
            // and the prefix is fetched from HBM once.  Otherwise equal contiguous
            // unit ranges (stream-K), two units or more per workgroup.
            long long s = pieces_for(pl.TP + wt);
            if (s >= 1) {
                const long long per = (pl.TP + wt) / s;       // a piece must not lie inside the booked units only
                if (wt > per) wt = per > 1 ? per : 1;
                s = pieces_for(pl.TP + wt);
            }
            pl.TPU = pl.TP + (int)wt;
            long long smax = NM > 0 ? kNumCU / NM : 0;
            if (smax > pl.TPU / 2) smax = pl.TPU / 2;
            if (s >= 1 && NM * smax * 5 >= (long long)kNumCU * 4) {
                w = NM * s;
                pl.uniform = (int)s;
            } else {
                // (ranges are short here: book at most two units, so that no range lies inside them only)
                if (wt > 2) wt = 2;
                pl.TPU = pl.TP + (int)wt;
                const long long U = NM * pl.TPU;
                w = U < 2 * kNumCU ? (U + 1) / 2 : kNumCU;
                if (w > U) w = U;
                if (w <= NM && NM <= kNumCU) {   // nothing to gain from cutting M-tiles: one workgroup each
                    w = NM;
                    pl.uniform = 1;
                }
            }
        }
        pl.U = NM * pl.TPU;
        pl.W = (int)w;
        pl.splits = 0;
        const long long upw = pl.U / pl.W;
        pl.max_seg = pl.uniform > 0 ? pl.uniform : (int)((pl.TPU + upw - 1) / upw) + 1;
        partials = pl.W != NM;
    } else {
        pl.TPU = pl.TP > 0 ? pl.TP : 1;
        pl.U = NM * pl.TPU;
        int s = p.splits;
        if (s == 0) {
            s = (int)(kNumCU / NM);
            if (s > 64) s = 64;
        }
        if (s > pl.TP) s = pl.TP;
        if (s < 1) s = 1;
        pl.splits = s;
        pl.W = 0;
        pl.uniform = 0;
        pl.max_seg = s;
        partials = s > 1;
    }
    if (partials) {
        const size_t prow = (size_t)NM * pl.max_seg * pl.mtile_rows;
        pl.ws_o_bytes = (prow * p.D * (p.dtype == FDD_BF16 ? 2 : sizeof(float)) + 255) & ~(size_t)255;
        pl.ws_ml_bytes = (prow * 2 * sizeof(float) + 255) & ~(size_t)255;
    } else {
        pl.ws_o_bytes = 0;
        pl.ws_ml_bytes = 0;
    }
    // The kernel reads V repacked when the caller brings it that way (fdd_prefix_pack, once per prefix).
    // Repacking inside the call is a launch and a pass over V of its own, and the kernel that reads V as it
    // lies (transposing LDS reads) is only about 2.5 % slower: measured, the in-call pass pays from about
    // the size of N=16, B=64, L=16384 on (28 M-tiles x 256 tiles per KV head), and costs 3..5 us below it.
    pl.ws_vt_bytes = 0;
    pl.packed = p.dtype == FDD_BF16 && p.L >= pl.key_tile && (p.prefix_v_packed || (long long)pl.MT * pl.TP >= 8192);
    if (pl.packed && !p.prefix_v_packed)
        pl.ws_vt_bytes = (((size_t)p.Hkv * batch * (p.L / pl.key_tile) * pl.key_tile * p.D * 2) + 255) & ~(size_t)255;
    *plan = pl;
    return true;
}

}  // namespace fdd

using namespace fdd;

static fdd_status check_unmask_shape(const fdd_unmask_params* p, const char* fn)
{
    if (!p) return fail(FDD_ERR_NULL, "%s: params is NULL", fn);
    if (p->N <= 0 || p->B <= 0 || p->V <= 0) return fail(FDD_ERR_SHAPE, "%s: N, B, V must be positive (got N=%d B=%d V=%lld)", fn, p->N, p->B, (long long)p->V);
    if (p->V >= (1ll << 31)) return fail(FDD_ERR_SHAPE, "%s: V must be below 2^31", fn);
    if ((long long)p->N * p->B > (1ll << 24)) return fail(FDD_ERR_SHAPE, "%s: N*B too large", fn);
    if (p->dtype != FDD_F32 && p->dtype != FDD_BF16) return fail(FDD_ERR_DTYPE, "%s: dtype %d is neither FDD_F32 nor FDD_BF16", fn, p->dtype);
    if (std::isnan(p->tau)) return fail(FDD_ERR_UNSUPPORTED, "%s: tau is NaN", fn);
    return FDD_OK;
}


// shape, type and pointer checks shared by the entry points of the unmask step (everything but the workspace)
fdd_status fdd::check_unmask_args(const fdd_unmask_params* p, const char* fn)
{
    fdd_status st = check_unmask_shape(p, fn);
    if (st != FDD_OK) return st;
    if (!p->logits || !p->mask || !p->tokens || !p->confidences)
        return fail(FDD_ERR_NULL, "%s: logits, mask, tokens and confidences must not be NULL", fn);
    if (!aligned16(p->logits)) return fail(FDD_ERR_UNSUPPORTED, "%s: logits must be 16-byte aligned", fn);
    if (p->refresh_table_k || p->refresh_table_v || p->refresh_block_k || p->refresh_block_v) {
        if (!p->refresh_table_k || !p->refresh_table_v || !p->refresh_block_k || !p->refresh_block_v)
            return fail(FDD_ERR_NULL, "%s: the K/V refresh needs refresh_table_k, refresh_table_v, refresh_block_k and refresh_block_v", fn);
        if (p->refresh_Hkv <= 0 || p->refresh_D <= 0 || p->refresh_T <= 0)
            return fail(FDD_ERR_SHAPE, "%s: refresh_Hkv, refresh_D, refresh_T must be positive", fn);
        if (p->refresh_dtype != FDD_F32 && p->refresh_dtype != FDD_BF16)
            return fail(FDD_ERR_DTYPE, "%s: refresh_dtype %d is neither FDD_F32 nor FDD_BF16", fn, p->refresh_dtype);
        const long long row = (long long)p->refresh_Hkv * p->refresh_D * (p->refresh_dtype == FDD_BF16 ? 2 : 4);
        if (row % 16 || row > (1ll << 24)) return fail(FDD_ERR_UNSUPPORTED, "%s: a refreshed K/V row must be a multiple of 16 bytes (and at most 16 MiB)", fn);
        if (!aligned16(p->refresh_table_k) || !aligned16(p->refresh_table_v) || !aligned16(p->refresh_block_k) || !aligned16(p->refresh_block_v))
            return fail(FDD_ERR_UNSUPPORTED, "%s: refresh tables and block K/V must be 16-byte aligned", fn);
    }
    return FDD_OK;
}

extern "C" {

size_t fdd_block_attn_workspace(const fdd_attn_params* p)
{
    if (check_attn_shape(p) != FDD_OK) return 0;
    AttnPlan plan;
    make_attn_plan(*p, &plan);
    return plan.ws_o_bytes + plan.ws_ml_bytes + plan.ws_vt_bytes;
}

fdd_status fdd_block_attn(const fdd_attn_params* p)
{
    fdd_status st = check_attn_shape(p);
    if (st != FDD_OK) return st;
    if (!p->q || !p->block_k || !p->block_v || !p->out) return fail(FDD_ERR_NULL, "fdd_block_attn: q, block_k, block_v and out must not be NULL");
    if (p->L > 0 && (!p->prefix_k || !p->prefix_v)) return fail(FDD_ERR_NULL, "fdd_block_attn: prefix_k / prefix_v is NULL with L=%d", p->L);
    if (p->E > 0 && (!p->ext_k || !p->ext_v)) return fail(FDD_ERR_NULL, "fdd_block_attn: ext_k / ext_v is NULL with E=%d", p->E);
    if (p->n_q_positions > 0 && !p->q_positions) return fail(FDD_ERR_NULL, "fdd_block_attn: q_positions is NULL with n_q_positions=%d", p->n_q_positions);
    if (p->n_q_positions > 0 && (reinterpret_cast<uintptr_t>(p->q_positions) & 3u)) return fail(FDD_ERR_UNSUPPORTED, "fdd_block_attn: q_positions must be 4-byte aligned");
    const void* ptrs[] = {p->q, p->prefix_k, p->prefix_v, p->block_k, p->block_v, p->out, p->prefix_v_packed,
                          p->E > 0 ? p->ext_k : nullptr, p->E > 0 ? p->ext_v : nullptr};
    for (const void* x : ptrs)
        if (x && !aligned16(x)) return fail(FDD_ERR_UNSUPPORTED, "fdd_block_attn: data pointers must be 16-byte aligned");
    if (p->out == p->q) return fail(FDD_ERR_UNSUPPORTED, "fdd_block_attn: out must not alias q");
    AttnPlan plan;
    make_attn_plan(*p, &plan);
    const size_t need = plan.ws_o_bytes + plan.ws_ml_bytes + plan.ws_vt_bytes;
    if (need > 0) {
        if (!p->workspace) return fail(FDD_ERR_WORKSPACE, "fdd_block_attn: workspace is NULL, %zu bytes needed", need);
        if (reinterpret_cast<uintptr_t>(p->workspace) & 255u) return fail(FDD_ERR_WORKSPACE, "fdd_block_attn: workspace must be 256-byte aligned");
        if (p->workspace_bytes < need) return fail(FDD_ERR_WORKSPACE, "fdd_block_attn: workspace has %zu bytes, %zu needed", p->workspace_bytes, need);
    }
    const float scale = p->scale > 0.f ? p->scale : 1.f / std::sqrt((float)p->D);
    hipStream_t s = static_cast<hipStream_t>(p->stream);
    const bool timed = g_ev_start && g_ev_stop;
    hipError_t e;
    if (p->dtype == FDD_BF16) {
        e = launch_attn_bf16(*p, plan, scale, s, timed ? g_ev_start : nullptr);
    } else {
        if (timed && hipEventRecord(g_ev_start, s) != hipSuccess) return fail(FDD_ERR_LAUNCH, "fdd_block_attn: cannot record the start event");
        e = launch_attn_f32(*p, plan, scale, s);
    }
    if (e != hipSuccess) return fail(FDD_ERR_LAUNCH, "fdd_block_attn: launch failed: %s", hipGetErrorString(e));
    if (timed && hipEventRecord(g_ev_stop, s) != hipSuccess) return fail(FDD_ERR_LAUNCH, "fdd_block_attn: cannot record the stop event");
    if (plan.ws_o_bytes > 0) {
        e = p->dtype == FDD_BF16 ? launch_attn_merge_bf16(*p, plan, scale, s) : launch_attn_combine(*p, plan, scale, s);
        if (e != hipSuccess) return fail(FDD_ERR_LAUNCH, "fdd_block_attn: merge launch failed: %s", hipGetErrorString(e));
    }
    return FDD_OK;
}

size_t fdd_prefix_pack_bytes(int32_t L, int32_t Hkv, int32_t D, int32_t dtype)
{
    if (dtype != FDD_BF16 || L < 64 || Hkv <= 0 || (D != 64 && D != 128)) return 0;
    return (((size_t)Hkv * (L / 64) * 64 * D * 2) + 255) & ~(size_t)255;
}

fdd_status fdd_prefix_pack(const void* prefix_v, int32_t L, int32_t Hkv, int32_t D, int32_t dtype, void* packed,
                           size_t packed_bytes, void* stream)
{
    if (dtype != FDD_BF16) return fail(FDD_ERR_DTYPE, "fdd_prefix_pack: only FDD_BF16 prefixes are packed");
    if (L < 0 || Hkv <= 0) return fail(FDD_ERR_SHAPE, "fdd_prefix_pack: L must be >= 0 and Hkv positive");
    if (D != 64 && D != 128) return fail(FDD_ERR_UNSUPPORTED, "fdd_prefix_pack: head size D=%d not supported (64 or 128)", D);
    if ((long long)L * Hkv >= (1ll << 31) || (long long)L * Hkv * D * 4 >= (1ll << 31))
        return fail(FDD_ERR_SHAPE, "fdd_prefix_pack: prefix V (L*Hkv*D elements) must stay below 2 GiB");
    const size_t need = fdd_prefix_pack_bytes(L, Hkv, D, dtype);
    if (need == 0) return FDD_OK;
    if (!prefix_v || !packed) return fail(FDD_ERR_NULL, "fdd_prefix_pack: prefix_v and packed must not be NULL");
    if (!aligned16(prefix_v) || !aligned16(packed)) return fail(FDD_ERR_UNSUPPORTED, "fdd_prefix_pack: pointers must be 16-byte aligned");
    if (packed_bytes < need) return fail(FDD_ERR_WORKSPACE, "fdd_prefix_pack: packed buffer has %zu bytes, %zu needed", packed_bytes, need);
    hipError_t e = launch_prefix_pack(prefix_v, L, Hkv, D, packed, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(FDD_ERR_LAUNCH, "fdd_prefix_pack: launch failed: %s", hipGetErrorString(e));
    return FDD_OK;
}

size_t fdd_unmask_workspace(const fdd_unmask_params* p)
{
    if (check_unmask_shape(p, "fdd_unmask_workspace") != FDD_OK) return 0;
    UnmaskPlan plan;
    make_unmask_plan(*p, &plan);
    return plan.ws_bytes;
}

fdd_status fdd_unmask_step(const fdd_unmask_params* p)
{
    fdd_status st = check_unmask_args(p, "fdd_unmask_step");
    if (st != FDD_OK) return st;
    UnmaskPlan plan;
    make_unmask_plan(*p, &plan);
    if (!p->workspace) return fail(FDD_ERR_WORKSPACE, "fdd_unmask_step: workspace is NULL, %zu bytes needed", plan.ws_bytes);
    if (reinterpret_cast<uintptr_t>(p->workspace) & 255u) return fail(FDD_ERR_WORKSPACE, "fdd_unmask_step: workspace must be 256-byte aligned");
    if (p->workspace_bytes < plan.ws_bytes) return fail(FDD_ERR_WORKSPACE, "fdd_unmask_step: workspace has %zu bytes, %zu needed", p->workspace_bytes, plan.ws_bytes);
    hipError_t e = launch_unmask(*p, plan, static_cast<hipStream_t>(p->stream));
    if (e != hipSuccess) return fail(FDD_ERR_LAUNCH, "fdd_unmask_step: launch failed: %s", hipGetErrorString(e));
    return FDD_OK;
}

size_t fdd_verify_workspace(const fdd_verify_params* p)
{
    UnmaskPlan plan;
    if (!p || p->V >= (1ll << 31) || (long long)p->N * p->B > (1ll << 24) ||
        (p->dtype != FDD_F32 && p->dtype != FDD_BF16) || !make_vocab_plan(p->N, p->B, p->V, p->dtype, !(p->temperature > 0.f), &plan))
        return 0;
    return plan.ws_bytes;
}

fdd_status fdd_verify_step(const fdd_verify_params* p)
{
    if (!p) return fail(FDD_ERR_NULL, "fdd_verify_step: params is NULL");
    if (p->N <= 0 || p->B <= 0 || p->V <= 0) return fail(FDD_ERR_SHAPE, "fdd_verify_step: N, B, V must be positive (got N=%d B=%d V=%lld)", p->N, p->B, (long long)p->V);
    if (p->V >= (1ll << 31)) return fail(FDD_ERR_SHAPE, "fdd_verify_step: V must be below 2^31");
    if ((long long)p->N * p->B > (1ll << 24)) return fail(FDD_ERR_SHAPE, "fdd_verify_step: N*B too large");
    if (p->dtype != FDD_F32 && p->dtype != FDD_BF16) return fail(FDD_ERR_DTYPE, "fdd_verify_step: dtype %d is neither FDD_F32 nor FDD_BF16", p->dtype);
    if (!(p->temperature >= 0.f) || std::isinf(p->temperature))
        return fail(FDD_ERR_UNSUPPORTED, "fdd_verify_step: temperature must be 0 (greedy) or positive and finite");
    if (!p->ar_logits || !p->draft || !p->mask || !p->tokens)
        return fail(FDD_ERR_NULL, "fdd_verify_step: ar_logits, draft, mask and tokens must not be NULL");
    if (!aligned16(p->ar_logits)) return fail(FDD_ERR_UNSUPPORTED, "fdd_verify_step: ar_logits must be 16-byte aligned");
    UnmaskPlan plan;
    make_vocab_plan(p->N, p->B, p->V, p->dtype, !(p->temperature > 0.f), &plan);
    if (!p->workspace) return fail(FDD_ERR_WORKSPACE, "fdd_verify_step: workspace is NULL, %zu bytes needed", plan.ws_bytes);
    if (reinterpret_cast<uintptr_t>(p->workspace) & 255u) return fail(FDD_ERR_WORKSPACE, "fdd_verify_step: workspace must be 256-byte aligned");
    if (p->workspace_bytes < plan.ws_bytes) return fail(FDD_ERR_WORKSPACE, "fdd_verify_step: workspace has %zu bytes, %zu needed", p->workspace_bytes, plan.ws_bytes);
    hipError_t e = launch_verify(*p, plan, static_cast<hipStream_t>(p->stream));
    if (e != hipSuccess) return fail(FDD_ERR_LAUNCH, "fdd_verify_step: launch failed: %s", hipGetErrorString(e));
    return FDD_OK;
}

fdd_status fdd_fork_block(int32_t N, size_t bytes, const void* src, void* dst, void* stream)
{
    if (!src || !dst) return fail(FDD_ERR_NULL, "fdd_fork_block: src and dst must not be NULL");
    if (N <= 0 || bytes == 0) return fail(FDD_ERR_SHAPE, "fdd_fork_block: N and bytes must be positive");
    if (bytes % 4 || (reinterpret_cast<uintptr_t>(src) & 3u) || (reinterpret_cast<uintptr_t>(dst) & 3u))
        return fail(FDD_ERR_UNSUPPORTED, "fdd_fork_block: bytes and pointers must be multiples of 4");
    if (bytes > (SIZE_MAX >> 1) / (size_t)N) return fail(FDD_ERR_SHAPE, "fdd_fork_block: N*bytes too large");
    const uintptr_t s0 = reinterpret_cast<uintptr_t>(src), d0 = reinterpret_cast<uintptr_t>(dst);
    const uintptr_t total = (uintptr_t)N * bytes;
    if (s0 > UINTPTR_MAX - bytes || d0 > UINTPTR_MAX - total) return fail(FDD_ERR_SHAPE, "fdd_fork_block: address range wraps around");
    if (s0 < d0 + total && d0 < s0 + bytes) return fail(FDD_ERR_UNSUPPORTED, "fdd_fork_block: src and dst overlap");
    hipError_t e = launch_fork_block(N, bytes, src, dst, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(FDD_ERR_LAUNCH, "fdd_fork_block: launch failed: %s", hipGetErrorString(e));
    return FDD_OK;
}

fdd_status fdd_block_commit(const fdd_commit_params* p)
{
    if (!p) return fail(FDD_ERR_NULL, "fdd_block_commit: params is NULL");
    if (p->N <= 0 || p->B <= 0 || p->Hkv <= 0 || p->D <= 0 || p->E < 0 || p->ext_capacity <= 0)
        return fail(FDD_ERR_SHAPE, "fdd_block_commit: N, B, Hkv, D, ext_capacity must be positive and E >= 0");
    if ((long long)p->E + p->B > p->ext_capacity)
        return fail(FDD_ERR_SHAPE, "fdd_block_commit: E + B = %lld exceeds ext_capacity = %d", (long long)p->E + p->B, p->ext_capacity);
    if (p->dtype != FDD_F32 && p->dtype != FDD_BF16) return fail(FDD_ERR_DTYPE, "fdd_block_commit: dtype %d is neither FDD_F32 nor FDD_BF16", p->dtype);
    if (p->reserved != 0) return fail(FDD_ERR_UNSUPPORTED, "fdd_block_commit: reserved field must be 0");
    if (!p->block_k || !p->block_v || !p->ext_k || !p->ext_v) return fail(FDD_ERR_NULL, "fdd_block_commit: block_k, block_v, ext_k and ext_v must not be NULL");
    const size_t es = p->dtype == FDD_BF16 ? 2 : 4;
    if (((size_t)p->Hkv * p->D * es) % 16) return fail(FDD_ERR_UNSUPPORTED, "fdd_block_commit: a K/V row must be a multiple of 16 bytes");
    const void* ptrs[] = {p->block_k, p->block_v, p->ext_k, p->ext_v};
    for (const void* x : ptrs)
        if (!aligned16(x)) return fail(FDD_ERR_UNSUPPORTED, "fdd_block_commit: pointers must be 16-byte aligned");
    hipError_t e = launch_block_commit(*p, static_cast<hipStream_t>(p->stream));
    if (e != hipSuccess) return fail(FDD_ERR_LAUNCH, "fdd_block_commit: launch failed: %s", hipGetErrorString(e));
    return FDD_OK;
}

fdd_status fdd_traj_mean(int32_t N, int32_t P, const float* traj, float* out, void* stream)
{
    if (!traj || !out) return fail(FDD_ERR_NULL, "fdd_traj_mean: traj and out must not be NULL");
    if (N <= 0 || P <= 0) return fail(FDD_ERR_SHAPE, "fdd_traj_mean: N and P must be positive (got N=%d P=%d)", N, P);
    if ((reinterpret_cast<uintptr_t>(traj) & 3u) || (reinterpret_cast<uintptr_t>(out) & 3u))
        return fail(FDD_ERR_UNSUPPORTED, "fdd_traj_mean: pointers must be 4-byte aligned");
    hipError_t e = launch_traj_mean(N, P, traj, out, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(FDD_ERR_LAUNCH, "fdd_traj_mean: launch failed: %s", hipGetErrorString(e));
    return FDD_OK;
}

fdd_status fdd_block_kv_update(const fdd_kv_update_params* p)
{
    if (!p) return fail(FDD_ERR_NULL, "fdd_block_kv_update: params is NULL");
    if (p->N <= 0 || p->B <= 0 || p->Hkv <= 0 || p->D <= 0 || p->T <= 0)
        return fail(FDD_ERR_SHAPE, "fdd_block_kv_update: N, B, Hkv, D, T must be positive");
    if (p->dtype != FDD_F32 && p->dtype != FDD_BF16) return fail(FDD_ERR_DTYPE, "fdd_block_kv_update: dtype %d is neither FDD_F32 nor FDD_BF16", p->dtype);
    if (!p->tokens || !p->committed || !p->table_k || !p->table_v || !p->block_k || !p->block_v)
        return fail(FDD_ERR_NULL, "fdd_block_kv_update: all pointers must be non-NULL");
    const size_t es = p->dtype == FDD_BF16 ? 2 : 4;
    if (((size_t)p->Hkv * p->D * es) % 16) return fail(FDD_ERR_UNSUPPORTED, "fdd_block_kv_update: a K/V row (Hkv*D elements) must be a multiple of 16 bytes");
    if (!aligned16(p->table_k) || !aligned16(p->table_v) || !aligned16(p->block_k) || !aligned16(p->block_v))
        return fail(FDD_ERR_UNSUPPORTED, "fdd_block_kv_update: tables and block K/V must be 16-byte aligned");
    hipError_t e = launch_kv_update(*p, static_cast<hipStream_t>(p->stream));
    if (e != hipSuccess) return fail(FDD_ERR_LAUNCH, "fdd_block_kv_update: launch failed: %s", hipGetErrorString(e));
    return FDD_OK;
}

fdd_status fdd_profile_attn_events(void* start, void* stop)
{
    if ((start == nullptr) != (stop == nullptr)) return fail(FDD_ERR_NULL, "fdd_profile_attn_events: pass two events or two NULLs");
    g_ev_start = static_cast<hipEvent_t>(start);
    g_ev_stop = static_cast<hipEvent_t>(stop);
    return FDD_OK;
}

const char* fdd_last_error(void) { return g_err; }

int fdd_version(void) { return 100; }

}  // extern "C"
