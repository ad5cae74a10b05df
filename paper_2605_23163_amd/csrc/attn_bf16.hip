// Shared-prefix block-causal attention, bf16 storage, gfx950 matrix cores.
//
// What is computed (paper, "Block-Causal Diffusion" and "Shared prefix"):
// every query row of every rollout attends to the L prefix keys and to the
// B keys of its own rollout's block.  Nothing here knows about layers or
// models; the prefix K/V is read through one pointer for all rollouts.
//
// How the work is laid out
//   * For one KV head, the query rows of all rollouts, block positions and
//     group heads are stacked into one list of R = N*B*G rows and cut into
//     M-tiles of 32 rows per wavefront.  Every prefix K/V tile a workgroup
//     stages in LDS is therefore used by all its stacked rows, whichever
//     rollout they come from; the prefix is never replicated.
//   * Scores are produced transposed, S^T = K Q^T, with the 32x32x16 bf16
//     MFMA: each lane then owns ONE query row (lane % 32) and 16 keys per
//     32-key block, so the row maximum and the row sum of the streaming
//     softmax are in-lane reductions plus a single exchange between the two
//     32-lane halves.  The same registers, rounded to bf16, are the B
//     operand of O^T += V^T P^T, so P never leaves the register file and the
//     accumulator keeps one query row per lane: its rescale is a per-lane
//     scalar multiply.
//   * V^T needs the key index contiguous per lane, so V tiles are transposed
//     on their way into LDS ([d][key], keys permuted so the 8 keys a lane
//     feeds to one MFMA are 16 contiguous bytes).  K tiles are stored
//     [key][d].  Both use a 16-byte row pad that makes the 128-bit fragment
//     reads bank-conflict free.
//   * The prefix is cut into `splits` pieces along L; each piece keeps the
//     streaming-softmax state (m, l, o) per row and writes it as an fp32
//     partial that a second small kernel merges (log-sum-exp merge).  With
//     one piece the kernel normalises and writes bf16 output directly.
//   * The in-block tail runs through the same tile loop: after the prefix
//     tiles, the workgroup stages the block K/V of each rollout its rows
//     belong to and masks the rows of other rollouts to -inf.
#include "fdd_internal.h"

namespace fdd {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;
typedef __attribute__((__vector_size__(2 * sizeof(uint32_t)))) uint32_t u32x2;

constexpr int KT = 64;           // keys per tile
constexpr int VROW = KT * 2 + 16;  // bytes per row of the transposed V tile

struct Args {
    const uint16_t* q;
    const uint16_t* pk;
    const uint16_t* pv;
    const uint16_t* bk;
    const uint16_t* bv;
    uint16_t* out;
    float* ws_o;
    float* ws_ml;
    int N, B, L, Hq, Hkv, G, R, MT, TP, S;
    float c;   // scale * log2(e)
};

// One 64-key tile of K and V to stream: where it starts, how many of its
// keys exist, and which rollout's rows may see it (-1: every row).
struct Tile {
    const uint16_t* k;
    const uint16_t* v;
    int valid;
    int rollout;
};

template <int D, int WAVES>
struct Cfg {
    static constexpr int THREADS = WAVES * 64;
    static constexpr int KROW = D * 2 + 16;             // bytes per K row in LDS
    static constexpr int K_BYTES = KT * KROW;
    static constexpr int V_BYTES = D * VROW;
    static constexpr int BUF_BYTES = K_BYTES + V_BYTES;
    static constexpr int K_CHUNKS = KT * (D / 8);        // 16-byte pieces of a K tile
    static constexpr int K_PER_THREAD = K_CHUNKS / THREADS;
    static constexpr int V_TASKS = (KT / 4) * (D / 2);   // (4 keys) x (2 channels) pieces
    static constexpr int V_PER_THREAD = V_TASKS / THREADS;
    static_assert(K_CHUNKS % THREADS == 0 && V_TASKS % THREADS == 0, "tile must divide over the workgroup");
};

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ float other_half(float x) { return __shfl_xor(x, 32, 64); }

template <int D, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void attn_bf16_kernel(Args a)
{
    using C = Cfg<D, WAVES>;
    constexpr int KS = D / 16;   // MFMA k-steps of Q K^T
    constexpr int DB = D / 32;   // 32-channel blocks of the output
    constexpr int MROWS = WAVES * 32;

    extern __shared__ __align__(16) unsigned char lds[];

    const int tid = threadIdx.x;
    const int wave = tid >> 6;
    const int lane = tid & 63;
    const int l32 = lane & 31;
    const int half = lane >> 5;

    // ---- which (kv head, M-tile, split) this workgroup owns ---------------
    // Workgroups are dealt to the 8 XCDs round-robin by their linear id.
    // All M-tiles that stream the same (head, split) piece of the prefix get
    // ids that are congruent modulo 8, hence the same XCD and the same L2.
    const int chunks = a.Hkv * a.S;
    const int xcd = blockIdx.x % kNumXCD;
    const int seq = blockIdx.x / kNumXCD;
    const int chunk = (seq / a.MT) * kNumXCD + xcd;
    const int mt = seq % a.MT;
    if (chunk >= chunks) return;
    const int kh = chunk / a.S;
    const int split = chunk % a.S;

    const int BG = a.B * a.G;
    const int row0_wg = mt * MROWS;
    const int row0 = row0_wg + wave * 32;
    const int row = row0 + l32;
    const bool row_ok = row < a.R;
    const int nb = row_ok ? row / a.G : 0;           // n*B + b
    const int g = row_ok ? row % a.G : 0;
    const int my_rollout = row_ok ? nb / a.B : -1;
    // rollouts spanned by this wave's rows and by the whole M-tile
    const int wave_n_lo = row0 / BG;
    const int wave_n_hi = (min(row0 + 31, a.R - 1)) / BG;
    const bool wave_has_rows = row0 < a.R;
    const int wg_n_lo = row0_wg / BG;
    const int wg_n_hi = (min(row0_wg + MROWS - 1, a.R - 1)) / BG;

    // ---- Q fragments: B operand of S^T = K Q^T ------------------------------
    bf16x8 qf[KS];
    {
        const uint16_t* qp = a.q + ((size_t)nb * a.Hq + (size_t)kh * a.G + g) * D + half * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            u32x4 raw = {0u, 0u, 0u, 0u};
            if (row_ok) raw = *reinterpret_cast<const u32x4*>(qp + ks * 16);
            qf[ks] = __builtin_bit_cast(bf16x8, raw);
        }
    }

    // ---- tile schedule -------------------------------------------------------
    const int t0 = (int)(((long long)split * a.TP) / a.S);
    const int t1 = (int)(((long long)(split + 1) * a.TP) / a.S);
    const int n_prefix = t1 - t0;
    const int tail_tiles_per_rollout = (a.B + KT - 1) / KT;
    const int n_tail = (split == a.S - 1) ? (wg_n_hi - wg_n_lo + 1) * tail_tiles_per_rollout : 0;
    const int n_tiles = n_prefix + n_tail;
    const size_t kv_stride = (size_t)a.Hkv * D;       // elements between consecutive keys

    auto tile_at = [&](int i) -> Tile {
        Tile t;
        if (i < n_prefix) {
            const int key0 = (t0 + i) * KT;
            t.k = a.pk + (size_t)key0 * kv_stride + (size_t)kh * D;
            t.v = a.pv + (size_t)key0 * kv_stride + (size_t)kh * D;
            t.valid = min(KT, a.L - key0);
            t.rollout = -1;
        } else {
            const int j = i - n_prefix;
            const int n = wg_n_lo + j / tail_tiles_per_rollout;
            const int key0 = (j % tail_tiles_per_rollout) * KT;
            const size_t off = ((size_t)n * a.B + key0) * kv_stride + (size_t)kh * D;
            t.k = a.bk + off;
            t.v = a.bv + off;
            t.valid = min(KT, a.B - key0);
            t.rollout = n;
        }
        return t;
    };

    // ---- global -> register staging of one tile -----------------------------
    u32x4 kreg[C::K_PER_THREAD];
    uint32_t vreg[C::V_PER_THREAD][4];

    auto load_tile = [&](const Tile& t) {
#pragma unroll
        for (int i = 0; i < C::K_PER_THREAD; ++i) {
            const int c = tid + i * C::THREADS;
            const int key = c / (D / 8);
            const int col = c % (D / 8);
            u32x4 x = {0u, 0u, 0u, 0u};
            if (key < t.valid) x = *reinterpret_cast<const u32x4*>(t.k + (size_t)key * kv_stride + col * 8);
            kreg[i] = x;
        }
#pragma unroll
        for (int i = 0; i < C::V_PER_THREAD; ++i) {
            const int task = tid + i * C::THREADS;
            const int dp = task % (D / 2);
            const int kg = task / (D / 2);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int key = kg * 4 + j;
                uint32_t x = 0u;
                if (key < t.valid) x = *reinterpret_cast<const uint32_t*>(t.v + (size_t)key * kv_stride + dp * 2);
                vreg[i][j] = x;
            }
        }
    };

    auto store_tile = [&](int buf) {
        unsigned char* kl = lds + buf * C::BUF_BYTES;
        unsigned char* vl = kl + C::K_BYTES;
#pragma unroll
        for (int i = 0; i < C::K_PER_THREAD; ++i) {
            const int c = tid + i * C::THREADS;
            const int key = c / (D / 8);
            const int col = c % (D / 8);
            *reinterpret_cast<u32x4*>(kl + key * C::KROW + col * 16) = kreg[i];
        }
#pragma unroll
        for (int i = 0; i < C::V_PER_THREAD; ++i) {
            const int task = tid + i * C::THREADS;
            const int dp = task % (D / 2);
            const int kg = task / (D / 2);
            // keys 4kg..4kg+3 of channels 2dp and 2dp+1 -> two 8-byte rows of V^T.
            // Key groups are stored with bits 0 and 1 of kg swapped, so that the
            // 8 keys one lane feeds to one MFMA k-step sit in 16 contiguous bytes.
            const int pg = (kg & ~3) | ((kg & 1) << 1) | ((kg & 2) >> 1);
            const uint32_t x0 = vreg[i][0], x1 = vreg[i][1], x2 = vreg[i][2], x3 = vreg[i][3];
            u32x2 even = {(x0 & 0xffffu) | (x1 << 16), (x2 & 0xffffu) | (x3 << 16)};
            u32x2 odd = {(x0 >> 16) | (x1 & 0xffff0000u), (x2 >> 16) | (x3 & 0xffff0000u)};
            unsigned char* p = vl + (2 * dp) * VROW + pg * 8;
            *reinterpret_cast<u32x2*>(p) = even;
            *reinterpret_cast<u32x2*>(p + VROW) = odd;
        }
    };

    // ---- streaming-softmax state: one query row per lane --------------------
    f32x16 o[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[db][v] = 0.f;
    float m_run = -INFINITY;   // running maximum of the raw scores
    float l_run = 0.f;         // this lane's share of the running sum

    auto compute_tile = [&](int buf, const Tile& t) {
        const unsigned char* kl = lds + buf * C::BUF_BYTES;
        const unsigned char* vl = kl + C::K_BYTES;
        f32x16 s[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
            for (int v = 0; v < 16; ++v) s[kb][v] = 0.f;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const bf16x8 kf = *reinterpret_cast<const bf16x8*>(kl + (kb * 32 + l32) * C::KROW + ks * 32 + half * 16);
                s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], s[kb], 0, 0, 0);
            }
        }
        // register v of block kb is key kb*32 + (v/4)*8 + half*4 + v%4
        const bool row_sees = (t.rollout < 0) || (t.rollout == my_rollout);
        if (t.valid < KT || t.rollout >= 0) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int key = kb * 32 + (v >> 2) * 8 + half * 4 + (v & 3);
                    if (!row_sees || key >= t.valid) s[kb][v] = -INFINITY;
                }
        }
        float mx = s[0][0];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v) mx = fmaxf(mx, s[kb][v]);
        mx = fmaxf(mx, other_half(mx));
        const float m_new = fmaxf(m_run, mx);
        const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = fast_exp2((m_run - m_use) * a.c);
        const float mc = m_use * a.c;
        float psum = 0.f;
        bf16x8 pf[4];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const float p = fast_exp2(fmaf(s[kb][v], a.c, -mc));
                psum += p;
                pf[kb * 2 + (v >> 3)][v & 7] = (__bf16)p;
            }
        l_run = l_run * alpha + psum;
        m_run = m_new;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int v = 0; v < 16; ++v) o[db][v] *= alpha;
#pragma unroll
        for (int t4 = 0; t4 < 4; ++t4)
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                const bf16x8 vf = *reinterpret_cast<const bf16x8*>(vl + (db * 32 + l32) * VROW + (t4 * 16 + half * 8) * 2);
                o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[t4], o[db], 0, 0, 0);
            }
    };

    // ---- main loop: double-buffered tiles ------------------------------------
    if (n_tiles > 0) {
        Tile cur = tile_at(0);
        load_tile(cur);
        store_tile(0);
        __syncthreads();
        for (int i = 0; i < n_tiles; ++i) {
            Tile nxt = cur;
            const bool more = i + 1 < n_tiles;
            if (more) {
                nxt = tile_at(i + 1);
                load_tile(nxt);
            }
            const bool wave_active = wave_has_rows &&
                (cur.rollout < 0 || (cur.rollout >= wave_n_lo && cur.rollout <= wave_n_hi));
            if (wave_active) compute_tile(i & 1, cur);
            if (more) store_tile((i + 1) & 1);
            __syncthreads();
            cur = nxt;
        }
    }

    // ---- epilogue -------------------------------------------------------------
    const float l_tot = l_run + other_half(l_run);
    if (!row_ok) return;
    if (a.S == 1) {
        const float inv = 1.f / l_tot;
        uint16_t* op = a.out + ((size_t)nb * a.Hq + (size_t)kh * a.G + g) * D;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4) {
                const int d = db * 32 + v4 * 8 + half * 4;
                typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
                bf16x4 w;
#pragma unroll
                for (int j = 0; j < 4; ++j) w[j] = (__bf16)(o[db][v4 * 4 + j] * inv);
                *reinterpret_cast<bf16x4*>(op + d) = w;
            }
    } else {
        const size_t prow = (((size_t)kh * a.MT + mt) * a.S + split) * MROWS + (wave * 32 + l32);
        float* wo = a.ws_o + prow * D;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4) {
                const int d = db * 32 + v4 * 8 + half * 4;
                float4 w = make_float4(o[db][v4 * 4 + 0], o[db][v4 * 4 + 1], o[db][v4 * 4 + 2], o[db][v4 * 4 + 3]);
                *reinterpret_cast<float4*>(wo + d) = w;
            }
        if (half == 0) {
            a.ws_ml[prow * 2 + 0] = m_run;
            a.ws_ml[prow * 2 + 1] = l_tot;
        }
    }
}

template <int D, int WAVES>
hipError_t launch(const Args& a, hipStream_t stream)
{
    using C = Cfg<D, WAVES>;
    const int chunks = a.Hkv * a.S;
    const int chunk_groups = (chunks + kNumXCD - 1) / kNumXCD;
    const int grid = chunk_groups * a.MT * kNumXCD;
    const size_t lds_bytes = 2 * (size_t)C::BUF_BYTES;
    auto kern = attn_bf16_kernel<D, WAVES>;
    static bool attr_done = false;   // per instantiation
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    hipLaunchKernelGGL(kern, dim3(grid), dim3(C::THREADS), lds_bytes, stream, a);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_attn_bf16(const fdd_attn_params& p, const AttnPlan& plan, float scale, hipStream_t s)
{
    Args a;
    a.q = static_cast<const uint16_t*>(p.q);
    a.pk = static_cast<const uint16_t*>(p.prefix_k);
    a.pv = static_cast<const uint16_t*>(p.prefix_v);
    a.bk = static_cast<const uint16_t*>(p.block_k);
    a.bv = static_cast<const uint16_t*>(p.block_v);
    a.out = static_cast<uint16_t*>(p.out);
    a.ws_o = static_cast<float*>(p.workspace);
    a.ws_ml = reinterpret_cast<float*>(static_cast<char*>(p.workspace) + plan.ws_o_bytes);
    a.N = p.N; a.B = p.B; a.L = p.L; a.Hq = p.Hq; a.Hkv = p.Hkv;
    a.G = plan.G; a.R = plan.R; a.MT = plan.MT; a.TP = plan.TP; a.S = plan.splits;
    a.c = scale * 1.4426950408889634f;
    if (plan.mtile_rows != 256) return hipErrorInvalidValue;
    return p.D == 128 ? launch<128, 8>(a, s) : launch<64, 8>(a, s);
}

}  // namespace fdd
