// Shared-prefix block-causal attention, fp32 storage and arithmetic, and the
// split merge used by both storage types.
//
// The fp32 path exists for exactness checks on small problems (the bf16
// matrix-core kernel is the performance path).  It computes the same thing
// (paper, "Block-Causal Diffusion" and "Shared prefix") with plain fp32 FMAs:
// a workgroup owns 16 stacked query rows of one KV head and one piece of the
// key range, stages 32-key K/V tiles in LDS, and keeps the streaming-softmax
// state (m, l, o) per row.
#include "fdd_internal.h"

namespace fdd {
namespace {

constexpr int KT = 32;     // keys per tile
constexpr int RT = 16;     // rows per workgroup
constexpr int THREADS = 256;

struct Args {
    const float* q;
    const float* pk;
    const float* pv;
    const float* bk;
    const float* bv;
    float* out;
    float* ws_o;
    float* ws_ml;
    const float* ek;   // per-rollout extension [N, Ecap, Hkv, D]
    const float* ev;
    int E, Ecap;
    int batch;         // independent problems in this launch; element strides between their arrays:
    long long q_bs, p_bs, b_bs, e_bs, o_bs;
    int N, B, L, Hq, Hkv, G, R, MT, TP, S;
    int causal;   // in-block keys are visible up to the query's own position only
    float c;   // scale * log2(e)
    const int32_t* qpos;   // stacked rows are the listed block positions only (ascending n*B + b), or nullptr: all of them
};

// block position n*B + b of entry `e` of the list of query positions (clamped into range), or e itself without a list
__device__ __forceinline__ int position_of(const int32_t* qpos, int e, int NB)
{
    return qpos ? min(max(qpos[e], 0), NB - 1) : e;
}

template <int D>
__global__ __launch_bounds__(THREADS) void attn_f32_kernel(Args a)
{
    constexpr int DP = D + 4;          // padded row length (floats), keeps float4 alignment
    constexpr int DPT = D / 16;        // output channels per thread
    __shared__ __align__(16) float qs[RT * DP];
    __shared__ __align__(16) float ks[KT * DP];
    __shared__ __align__(16) float vs[KT * DP];
    __shared__ float ps[RT * (KT + 1)];

    const int tid = threadIdx.x;
    const int mt = blockIdx.x;
    const int split = blockIdx.y;
    // grid z runs over (problem of the batch, KV head); the pointers are moved to the problem's arrays
    const int khv = blockIdx.z;
    const int pb = khv / a.Hkv;
    const int kh = khv - pb * a.Hkv;
    a.q += pb * a.q_bs;
    a.pk += pb * a.p_bs;
    a.pv += pb * a.p_bs;
    a.bk += pb * a.b_bs;
    a.bv += pb * a.b_bs;
    a.ek += pb * a.e_bs;
    a.ev += pb * a.e_bs;
    a.out += pb * a.o_bs;
    const int BG = a.B * a.G;

    const int r_loc = tid / 16;         // row of this thread inside the workgroup tile
    const int sub = tid % 16;           // 16 threads cooperate on a row
    const int row = mt * RT + r_loc;
    const bool row_ok = row < a.R;
    const int NB = a.N * a.B;
    const int nb = row_ok ? position_of(a.qpos, row / a.G, NB) : 0;
    const int g = row_ok ? row % a.G : 0;
    const int my_rollout = row_ok ? nb / a.B : -1;
    const int my_b = row_ok ? nb % a.B : 0;
    // (rows are in ascending order of position, hence of rollout)
    const int wg_row_hi = min(mt * RT + RT - 1, a.R - 1);
    const int wg_n_lo = a.qpos ? position_of(a.qpos, (mt * RT) / a.G, NB) / a.B : (mt * RT) / BG;
    const int wg_n_hi = a.qpos ? position_of(a.qpos, wg_row_hi / a.G, NB) / a.B : wg_row_hi / BG;

    // stage the query rows
    for (int i = tid; i < RT * (D / 4); i += THREADS) {
        const int r = i / (D / 4), c4 = i % (D / 4);
        const int rr = mt * RT + r;
        float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
        if (rr < a.R) {
            const int nb_ = position_of(a.qpos, rr / a.G, NB), g_ = rr % a.G;
            x = *reinterpret_cast<const float4*>(a.q + ((size_t)nb_ * a.Hq + (size_t)kh * a.G + g_) * D + c4 * 4);
        }
        *reinterpret_cast<float4*>(&qs[r * DP + c4 * 4]) = x;
    }

    const int t0 = (int)(((long long)split * a.TP) / a.S);
    const int t1 = (int)(((long long)(split + 1) * a.TP) / a.S);
    const int n_prefix = t1 - t0;
    const int ext_per = (a.E + KT - 1) / KT;                  // tiles of a rollout's extension
    const int tail_per = ext_per + (a.B + KT - 1) / KT;       // private tiles per rollout: extension, then block
    const int n_tail = (split == a.S - 1) ? (wg_n_hi - wg_n_lo + 1) * tail_per : 0;
    const size_t kv_stride = (size_t)a.Hkv * D;

    float o[DPT];
#pragma unroll
    for (int j = 0; j < DPT; ++j) o[j] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    for (int i = 0; i < n_prefix + n_tail; ++i) {
        const float *kp, *vp;
        int valid, rollout, blk0 = 0;
        bool in_block = false;
        if (i < n_prefix) {
            const int key0 = (t0 + i) * KT;
            kp = a.pk + (size_t)key0 * kv_stride + (size_t)kh * D;
            vp = a.pv + (size_t)key0 * kv_stride + (size_t)kh * D;
            valid = min(KT, a.L - key0);
            rollout = -1;
        } else {
            const int j = i - n_prefix;
            const int n = wg_n_lo + j / tail_per;
            const int w = j % tail_per;
            rollout = n;
            if (w < ext_per) {
                const int key0 = w * KT;
                const size_t off = ((size_t)n * a.Ecap + key0) * kv_stride + (size_t)kh * D;
                kp = a.ek + off;
                vp = a.ev + off;
                valid = min(KT, a.E - key0);
            } else {
                const int key0 = (w - ext_per) * KT;
                const size_t off = ((size_t)n * a.B + key0) * kv_stride + (size_t)kh * D;
                kp = a.bk + off;
                vp = a.bv + off;
                valid = min(KT, a.B - key0);
                blk0 = key0;
                in_block = true;
            }
        }
        __syncthreads();   // previous tile fully consumed (and qs written, first time)
        for (int x = tid; x < KT * (D / 4); x += THREADS) {
            const int key = x / (D / 4), c4 = x % (D / 4);
            float4 kk = make_float4(0.f, 0.f, 0.f, 0.f), vv = kk;
            if (key < valid) {
                kk = *reinterpret_cast<const float4*>(kp + (size_t)key * kv_stride + c4 * 4);
                vv = *reinterpret_cast<const float4*>(vp + (size_t)key * kv_stride + c4 * 4);
            }
            *reinterpret_cast<float4*>(&ks[key * DP + c4 * 4]) = kk;
            *reinterpret_cast<float4*>(&vs[key * DP + c4 * 4]) = vv;
        }
        __syncthreads();

        // scores of KT/16 keys per thread: keys sub, sub+16, ...
        const bool sees = rollout < 0 || rollout == my_rollout;
        constexpr int KPT = KT / 16;
        float sc[KPT];
        float mx = -INFINITY;
#pragma unroll
        for (int j = 0; j < KPT; ++j) {
            const int key = sub + 16 * j;
            float acc = 0.f;
            for (int d = 0; d < D; d += 4) {
                const float4 qq = *reinterpret_cast<const float4*>(&qs[r_loc * DP + d]);
                const float4 kk = *reinterpret_cast<const float4*>(&ks[key * DP + d]);
                acc = fmaf(qq.x, kk.x, acc);
                acc = fmaf(qq.y, kk.y, acc);
                acc = fmaf(qq.z, kk.z, acc);
                acc = fmaf(qq.w, kk.w, acc);
            }
            const bool later = a.causal && in_block && blk0 + key > my_b;
            sc[j] = (sees && key < valid && !later) ? acc : -INFINITY;
            mx = fmaxf(mx, sc[j]);
        }
#pragma unroll
        for (int w = 8; w >= 1; w >>= 1) mx = fmaxf(mx, __shfl_xor(mx, w, 16));
        const float m_new = fmaxf(m_run, mx);
        const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = exp2f((m_run - m_use) * a.c);
        float psum = 0.f;
#pragma unroll
        for (int j = 0; j < KPT; ++j) {
            const float p = exp2f((sc[j] - m_use) * a.c);
            psum += p;
            ps[r_loc * (KT + 1) + sub + 16 * j] = p;
        }
#pragma unroll
        for (int w = 8; w >= 1; w >>= 1) psum += __shfl_xor(psum, w, 16);
        l_run = l_run * alpha + psum;
        m_run = m_new;
        __syncthreads();   // ps visible to the 16 threads of the row
#pragma unroll
        for (int j = 0; j < DPT; ++j) o[j] *= alpha;
        for (int key = 0; key < KT; ++key) {
            const float p = ps[r_loc * (KT + 1) + key];
#pragma unroll
            for (int j = 0; j < DPT; ++j) o[j] = fmaf(p, vs[key * DP + sub * DPT + j], o[j]);
        }
    }

    if (!row_ok) return;
    if (a.S == 1) {
        float* op = a.out + ((size_t)nb * a.Hq + (size_t)kh * a.G + g) * D + sub * DPT;
        const float inv = 1.f / l_run;
#pragma unroll
        for (int j = 0; j < DPT; ++j) op[j] = o[j] * inv;
    } else {
        const size_t prow = (((size_t)khv * a.MT + mt) * a.S + split) * RT + r_loc;
        float* wo = a.ws_o + prow * D + sub * DPT;
#pragma unroll
        for (int j = 0; j < DPT; ++j) wo[j] = o[j];
        if (sub == 0) {
            a.ws_ml[prow * 2 + 0] = m_run;
            a.ws_ml[prow * 2 + 1] = l_run;
        }
    }
}

// ---------------------------------------------------------------------------
// Merge of the per-segment partials (log-sum-exp merge), for both storage types:
//   m* = max_s m_s,  w_s = 2^((m_s - m*) c),  out = sum_s w_s o_s / sum_s w_s l_s
// The sum runs over s in a fixed order, so results are reproducible.
struct CombineArgs {
    const float* ws_o;
    const float* ws_ml;
    void* out;
    int Hq, Hkv, G, R, MT, mrows, D, bf16;
    long long o_bs;  // elements between the outputs of the problems of a batch
    int max_seg;     // slots per M-tile in the workspace
    int fixed_seg;   // > 0: every M-tile has this many segments; 0: stream-K ranges
    int TPU, base, rem;
    int SG;          // segment groups: the segments of a row are shared out over SG threads per channel quad
    int RB;          // rows per block; RB * SG * D/4 = 256 threads
    float c;
    const int32_t* qpos;   // list of query positions, as in the attention kernels, or nullptr
    int NB;                // N * B
};

// grid (Hkv*MT, ceil(mrows / RB)).  Thread (r, sg, d4) sums segments sg, sg+SG, ..
// of row r for 4 channels, four loads in flight at a time; the SG partial sums
// are then added in the order sg = 0, 1, .. by the thread with sg = 0.
__global__ __launch_bounds__(256) void attn_combine_kernel(CombineArgs a)
{
    extern __shared__ __align__(16) float smem[];
    const int d4n = a.D / 4;
    const int tid = (int)threadIdx.x;
    const int d4 = tid % d4n, sg = (tid / d4n) % a.SG, r = tid / (d4n * a.SG);
    const int M = (int)blockIdx.x;
    const int khv = M / a.MT, mt = M - khv * a.MT;      // (problem of the batch, KV head), M-tile
    const int pb = khv / a.Hkv, kh = khv - pb * a.Hkv;
    const int rit0 = (int)blockIdx.y * a.RB;
    int n_seg = a.fixed_seg;
    if (n_seg == 0) {
        // same arithmetic as the attention kernel: workgroups whose unit range meets this M-tile
        n_seg = wg_of_unit((M + 1) * a.TPU - 1, a.base, a.rem) - wg_of_unit(M * a.TPU, a.base, a.rem) + 1;
    }
    if (n_seg == 1) return;     // written in final form by its only segment
    if (a.SG == 1 && n_seg <= 4) {
        // few segments: every thread reads the (m, l) pairs of its row itself, together with its
        // partial outputs, in one round trip to memory and without LDS (same sums, same order)
        const int rit = rit0 + r;
        const int row = mt * a.mrows + rit;
        if (rit >= a.mrows || row >= a.R) return;
        const size_t prow = ((size_t)M * a.max_seg) * a.mrows + rit;
        float2 ml[4];
        float4 x[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            ml[u] = make_float2(-INFINITY, 0.f);
            x[u] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (u < n_seg) {
                ml[u] = *reinterpret_cast<const float2*>(a.ws_ml + (prow + (size_t)u * a.mrows) * 2);
                x[u] = *reinterpret_cast<const float4*>(a.ws_o + (prow + (size_t)u * a.mrows) * a.D + d4 * 4);
            }
        }
        float mstar = -INFINITY;
#pragma unroll
        for (int u = 0; u < 4; ++u) mstar = fmaxf(mstar, ml[u].x);
        float l = 0.f;
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (u < n_seg) {
                const float w = exp2f((ml[u].x - mstar) * a.c);
                l = fmaf(ml[u].y, w, l);
                acc.x = fmaf(x[u].x, w, acc.x);
                acc.y = fmaf(x[u].y, w, acc.y);
                acc.z = fmaf(x[u].z, w, acc.z);
                acc.w = fmaf(x[u].w, w, acc.w);
            }
        }
        const float inv = 1.f / l;
        const int sel = row / a.G, g = row - sel * a.G;
        const int nb = position_of(a.qpos, sel, a.NB);
        const size_t off = (size_t)(pb * a.o_bs) + ((size_t)nb * a.Hq + (size_t)kh * a.G + g) * a.D + d4 * 4;
        if (a.bf16) {
            typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
            bf16x4 w4;
            w4[0] = (__bf16)(acc.x * inv);
            w4[1] = (__bf16)(acc.y * inv);
            w4[2] = (__bf16)(acc.z * inv);
            w4[3] = (__bf16)(acc.w * inv);
            *reinterpret_cast<bf16x4*>(static_cast<uint16_t*>(a.out) + off) = w4;
        } else {
            *reinterpret_cast<float4*>(static_cast<float*>(a.out) + off) =
                make_float4(acc.x * inv, acc.y * inv, acc.z * inv, acc.w * inv);
        }
        return;
    }
    float* const sm = smem;                           // [RB][n_seg] segment maxima
    float* const sl = smem + a.RB * n_seg;            // [RB][n_seg] segment sums
    float4* const red = reinterpret_cast<float4*>(smem + ((2 * a.RB * a.max_seg + 3) & ~3));   // [RB][SG][d4n]
    float* const redl = reinterpret_cast<float*>(red + a.RB * a.SG * d4n);        // [RB][SG]
    const size_t p0 = ((size_t)M * a.max_seg) * a.mrows + rit0;
    for (int i = tid; i < a.RB * n_seg; i += 256) {
        const int rr = i / n_seg, s = i - rr * n_seg;
        float m = -INFINITY, l = 0.f;
        if (rit0 + rr < a.mrows) {
            const float2 ml = *reinterpret_cast<const float2*>(a.ws_ml + (p0 + rr + (size_t)s * a.mrows) * 2);
            m = ml.x;
            l = ml.y;
        }
        sm[i] = m;
        sl[i] = l;
    }
    __syncthreads();
    const int rit = rit0 + r;
    const int row = mt * a.mrows + rit;
    const bool live = rit < a.mrows && row < a.R;
    float mstar = -INFINITY;
    for (int s = 0; s < n_seg; ++s) mstar = fmaxf(mstar, sm[r * n_seg + s]);
    float l = 0.f;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    if (live) {
        const float* src = a.ws_o + (p0 + r) * a.D + d4 * 4;
        const size_t seg_stride = (size_t)a.mrows * a.D;
        for (int s0 = sg; s0 < n_seg; s0 += 4 * a.SG) {
            float4 x[4];
            float w[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int s = s0 + u * a.SG;
                x[u] = make_float4(0.f, 0.f, 0.f, 0.f);
                w[u] = 0.f;
                if (s < n_seg) {
                    x[u] = *reinterpret_cast<const float4*>(src + (size_t)s * seg_stride);
                    w[u] = exp2f((sm[r * n_seg + s] - mstar) * a.c);
                    l = fmaf(sl[r * n_seg + s], w[u], l);
                }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                acc.x = fmaf(x[u].x, w[u], acc.x);
                acc.y = fmaf(x[u].y, w[u], acc.y);
                acc.z = fmaf(x[u].z, w[u], acc.z);
                acc.w = fmaf(x[u].w, w[u], acc.w);
            }
        }
    }
    if (a.SG > 1) {
        red[(r * a.SG + sg) * d4n + d4] = acc;
        if (d4 == 0) redl[r * a.SG + sg] = l;
        __syncthreads();
        if (sg != 0) return;
        acc = red[(r * a.SG) * d4n + d4];
        l = redl[r * a.SG];
        for (int k = 1; k < a.SG; ++k) {
            const float4 y = red[(r * a.SG + k) * d4n + d4];
            acc.x += y.x;
            acc.y += y.y;
            acc.z += y.z;
            acc.w += y.w;
            l += redl[r * a.SG + k];
        }
    }
    if (!live) return;
    const float inv = 1.f / l;
    const int sel = row / a.G, g = row - sel * a.G;
    const int nb = position_of(a.qpos, sel, a.NB);
    const size_t off = (size_t)(pb * a.o_bs) + ((size_t)nb * a.Hq + (size_t)kh * a.G + g) * a.D + d4 * 4;
    if (a.bf16) {
        typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
        bf16x4 w;
        w[0] = (__bf16)(acc.x * inv);
        w[1] = (__bf16)(acc.y * inv);
        w[2] = (__bf16)(acc.z * inv);
        w[3] = (__bf16)(acc.w * inv);
        *reinterpret_cast<bf16x4*>(static_cast<uint16_t*>(a.out) + off) = w;
    } else {
        *reinterpret_cast<float4*>(static_cast<float*>(a.out) + off) =
            make_float4(acc.x * inv, acc.y * inv, acc.z * inv, acc.w * inv);
    }
}

}  // namespace

hipError_t launch_attn_f32(const fdd_attn_params& p, const AttnPlan& plan, float scale, hipStream_t s)
{
    Args a;
    a.q = static_cast<const float*>(p.q);
    a.pk = static_cast<const float*>(p.prefix_k);
    a.pv = static_cast<const float*>(p.prefix_v);
    a.bk = static_cast<const float*>(p.block_k);
    a.bv = static_cast<const float*>(p.block_v);
    a.out = static_cast<float*>(p.out);
    a.ws_o = static_cast<float*>(p.workspace);
    a.ws_ml = reinterpret_cast<float*>(static_cast<char*>(p.workspace) + plan.ws_o_bytes);
    a.ek = static_cast<const float*>(p.ext_k);
    a.ev = static_cast<const float*>(p.ext_v);
    a.E = p.E; a.Ecap = p.ext_capacity;
    a.batch = p.batch > 1 ? p.batch : 1;
    a.q_bs = p.q_batch_stride; a.p_bs = p.prefix_batch_stride; a.b_bs = p.block_batch_stride;
    a.e_bs = p.ext_batch_stride; a.o_bs = p.out_batch_stride;
    a.N = p.N; a.B = p.B; a.L = p.L; a.Hq = p.Hq; a.Hkv = p.Hkv;
    a.G = plan.G; a.R = plan.R; a.MT = plan.MT; a.TP = plan.TP; a.S = plan.splits;
    a.c = scale * 1.4426950408889634f;
    a.causal = (p.flags & FDD_ATTN_CAUSAL_BLOCK) ? 1 : 0;
    a.qpos = p.n_q_positions > 0 ? p.q_positions : nullptr;
    if (plan.mtile_rows != RT) return hipErrorInvalidValue;
    const dim3 grid(plan.MT, plan.splits, p.Hkv * a.batch);
    if (p.D == 128) hipLaunchKernelGGL(attn_f32_kernel<128>, grid, dim3(THREADS), 0, s, a);
    else hipLaunchKernelGGL(attn_f32_kernel<64>, grid, dim3(THREADS), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_attn_combine(const fdd_attn_params& p, const AttnPlan& plan, float scale, hipStream_t s)
{
    CombineArgs a;
    a.ws_o = static_cast<const float*>(p.workspace);
    a.ws_ml = reinterpret_cast<const float*>(static_cast<const char*>(p.workspace) + plan.ws_o_bytes);
    a.out = p.out;
    const int batch = p.batch > 1 ? p.batch : 1;
    a.Hq = p.Hq; a.Hkv = p.Hkv; a.G = plan.G; a.R = plan.R; a.MT = plan.MT;
    a.o_bs = p.out_batch_stride;
    a.qpos = p.n_q_positions > 0 ? p.q_positions : nullptr;
    a.NB = p.N * p.B;
    a.mrows = plan.mtile_rows; a.D = p.D; a.bf16 = (p.dtype == FDD_BF16);
    a.max_seg = plan.max_seg;
    a.fixed_seg = a.bf16 ? plan.uniform : plan.splits;
    a.TPU = plan.TPU;
    a.base = a.bf16 ? (int)(plan.U / plan.W) : 1;
    a.rem = a.bf16 ? (int)(plan.U % plan.W) : 0;
    a.c = scale * 1.4426950408889634f;
    // more threads per row when the rows are few and the segments many
    const long long rows = (long long)p.Hkv * batch * plan.R;
    const int seg_hint = a.fixed_seg > 0 ? a.fixed_seg : plan.max_seg;
    int sg = 1;
    while (sg < 8 && sg * 2 <= seg_hint && rows * sg < 16384) sg *= 2;
    a.SG = sg;
    a.RB = 256 / (sg * (p.D / 4));
    const size_t smem = (size_t)((2 * a.RB * plan.max_seg + 3) & ~3) * sizeof(float) + (size_t)a.RB * sg * (p.D / 4) * sizeof(float4) +
                        (size_t)a.RB * sg * sizeof(float);
    if (smem > 60 * 1024) return hipErrorInvalidValue;
    const dim3 grid(p.Hkv * batch * plan.MT, (plan.mtile_rows + a.RB - 1) / a.RB);
    hipLaunchKernelGGL(attn_combine_kernel, grid, dim3(256), smem, s, a);
    return hipGetLastError();
}

}  // namespace fdd
