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
//   * O^T += V^T P^T needs, per lane, 8 keys of one channel, i.e. V with the
//     key index contiguous, while V lies in memory [key][d].  When an M-tile's
//     keys are streamed by more than one workgroup (R > 256 rows per KV head),
//     a small pre-pass packs the full prefix tiles of V once into the exact
//     fragment order, [tile][16-key step][half][d][8 keys], so the main kernel
//     moves those 16 KB tiles straight from global memory into LDS
//     (buffer_load ... lds, no registers, no vector ALU work) and reads
//     fragments as plain conflict-free 128-bit loads.  K tiles take the same
//     direct path, [key][d] with the 16-byte pieces of a row XOR-swizzled by
//     the row index, which keeps the K fragment reads conflict-free without
//     padding.  Otherwise (a single M-tile per head, the ragged last prefix
//     tile, the in-block tail) tiles are staged through registers as they lie
//     in memory and V^T fragments come from the gfx950 LDS transpose read
//     (ds_read_b64_tr_b16: lane i of a 16-lane group receives column i of a
//     4 x 16 block, i.e. 4 consecutive keys of channel i); row pads of 16
//     bytes (K) and 64 bytes (V) make both kinds of read conflict-free.
//   * Full prefix tiles run through a software-pipelined loop written as 32
//     slots per tile, one per MFMA.  Each slot also carries a slice of vector
//     ALU work that does not depend on that MFMA: while the matrix pipe
//     produces the scores of tile i+1 and then the P V products of tile i,
//     the vector ALUs reduce the row maximum of tile i, take its exponentials
//     and round them to bf16.  One wavefront can only issue a vector
//     instruction every other issue slot, so two wavefronts per SIMD running
//     this same mix are what fills both pipes.  K runs one tile ahead of V in
//     LDS (two buffers each), global loads another tile ahead in registers,
//     and LDS fragments are requested two MFMAs before their use.
//   * The softmax reference value of a row is only raised when the running
//     maximum outgrows it by more than 2^8; in between probabilities may
//     exceed 1, which fp32 sums and bf16 relative precision do not mind, and
//     the accumulator rescale becomes a rare wave-uniform branch.  The result
//     is mathematically the same softmax.
//   * Work is dealt out stream-K style.  The unit of work is one 64-key prefix
//     tile of one M-tile; all units, ordered by (KV head, M-tile, tile), are
//     cut into W equal contiguous ranges, one per workgroup, so every compute
//     unit gets the same amount of work whatever the shape.  A range may end
//     inside an M-tile and continue in the next one: each such segment keeps
//     its own streaming-softmax state (m, l, o) per row.  An M-tile that was
//     covered by a single segment is normalised and written as bf16 output
//     directly; otherwise the segments leave fp32 partials that a second small
//     kernel merges (log-sum-exp merge, fixed order).
//   * A ragged last prefix tile and the in-block tail go through a simpler
//     masked path: the workgroup stages the block K/V of each rollout its
//     rows belong to and masks the rows of other rollouts to -inf.
#include <type_traits>

#include "fdd_internal.h"

namespace fdd {
namespace attn_bf16 {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;
typedef __attribute__((__vector_size__(2 * sizeof(uint32_t)))) uint32_t u32x2;

constexpr int KT = 64;           // keys per tile
typedef short i16x4 __attribute__((ext_vector_type(4)));

struct Args {
    const uint16_t* q;
    const uint16_t* pk;
    const uint16_t* pv;
    const uint16_t* bk;
    const uint16_t* bv;
    uint16_t* out;
    float* ws_o;
    float* ws_ml;
    const uint16_t* vt;   // packed V^T tiles of the full prefix tiles (PACKED kernels only)
    int N, B, L, Hq, Hkv, G, R, MT, TP;
    int TPF;        // full prefix tiles = L / 64
    int TPU;        // units per M-tile = max(TP, 1)
    int W;          // workgroups
    int max_seg;    // partial slots per M-tile
    int S;          // > 0: every M-tile is cut into S equal pieces (W = Hkv*MT*S); 0: free ranges
    int causal;     // in-block keys are visible up to the query's own position only
    long long U;    // units in total = Hkv * MT * TPU
    float c;        // scale * log2(e)
};

// Segments of M-tile M: the workgroups whose unit range [U w / W, U (w+1) / W)
// meets [M TPU, (M+1) TPU).
__host__ __device__ inline int first_wg_of(long long M, const int TPU, const int W, const long long U)
{
    return (int)(((M * TPU + 1) * W + U - 1) / U) - 1;
}
__host__ __device__ inline int last_wg_of(long long M, const int TPU, const int W, const long long U)
{
    return (int)(((M + 1) * TPU * W + U - 1) / U) - 1;
}

// One 64-key tile of K and V to stream: where it starts, how many of its
// keys exist, and which rollout's rows may see it (-1: every row).
struct Tile {
    const uint16_t* k;
    const uint16_t* v;
    int valid;
    int rollout;
    int key0;   // block position of the tile's first key (tail tiles)
};

template <int D, int WAVES>
struct Cfg {
    static constexpr int THREADS = WAVES * 64;
    static constexpr int KROW = D * 2 + 16;             // bytes per K row in LDS
    static constexpr int VROW = D * 2 + 64;             // bytes per V row in LDS
    static constexpr int K_BYTES = KT * KROW;
    static constexpr int V_BYTES = KT * VROW;
    static constexpr int BUF_BYTES = K_BYTES + V_BYTES;
    static constexpr int K_CHUNKS = KT * (D / 8);        // 16-byte pieces of a K tile
    static constexpr int K_PER_THREAD = K_CHUNKS / THREADS;
    static_assert(K_CHUNKS % THREADS == 0, "tile must divide over the workgroup");
    // direct-to-LDS path: unpadded 64 x D tiles moved in 1 KB pieces, one per wavefront instruction
    static constexpr int T_BYTES = KT * D * 2;
    static constexpr int NI = T_BYTES / 1024 / WAVES;    // pieces per wavefront
    static constexpr int CH = D / 8;                     // 16-byte pieces per K row
    static constexpr int RPB = 1024 / (D * 2);           // K rows per 1 KB piece
    static constexpr int RPL = 256 / (D * 2);            // K rows per 256-byte bank line
    static_assert(NI >= 1 && T_BYTES % (1024 * WAVES) == 0, "tile must divide over the wavefronts");
};

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// value held by the lane 32 positions away (the other half of the wavefront)
__device__ __forceinline__ float other_half(float x)
{
    const unsigned u = __builtin_bit_cast(unsigned, x);
    // swaps lanes 32..63 of the first operand with lanes 0..31 of the second
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return __builtin_bit_cast(float, (threadIdx.x & 32) ? r[0] : r[1]);
}

// Nothing is scheduled across this point: the source order of the pieces it
// separates is the order the hardware sees.
#define FDD_SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)
// Forces a value to exist at this point of the instruction stream, so that
// the vector work of a slot is not sunk towards its first use.
#define FDD_PIN(x) asm volatile("" : "+v"(x))

template <int D, int WAVES, bool PACKED>
__global__ __launch_bounds__(WAVES * 64) void attn_bf16_kernel(Args a)
{
#if defined(__HIP_DEVICE_COMPILE__)   // the host pass only needs the launch stub
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

    // ---- stream-K: this workgroup's contiguous range of (M-tile, prefix tile) units
    // Workgroups are dealt to the 8 XCDs round-robin by their launch index.
    // Ranges are numbered so that the workgroups of one XCD own neighbouring
    // ranges.
    const int per_xcd = (a.W + kNumXCD - 1) / kNumXCD;
    int wg = (int)(blockIdx.x % kNumXCD) * per_xcd + (int)(blockIdx.x / kNumXCD);
    if (wg >= a.W) return;
    if (a.S > 0) {
        // equal pieces: neighbours are the M-tiles of one (KV head, piece), which
        // walk the same keys in step, so each XCD fetches its share of K/V once
        const int mt_ = wg % a.MT, piece = (wg / a.MT) % a.S, kh_ = wg / (a.MT * a.S);
        wg = (kh_ * a.MT + mt_) * a.S + piece;
    }
    const long long u_end = a.U * (wg + 1) / a.W;
    for (long long u_cur = a.U * wg / a.W; u_cur < u_end;) {
    const int M = (int)(u_cur / a.TPU);              // M-tile index over all KV heads
    const int t_begin = (int)(u_cur % a.TPU);
    const int t_end = (int)min((long long)a.TPU, t_begin + (u_end - u_cur));
    u_cur += t_end - t_begin;
    const int kh = M / a.MT;
    const int mt = M % a.MT;
    const int seg_first = first_wg_of(M, a.TPU, a.W, a.U);
    const int n_seg = last_wg_of(M, a.TPU, a.W, a.U) - seg_first + 1;
    const int seg = wg - seg_first;

    const int BG = a.B * a.G;
    const int row0_wg = mt * MROWS;
    const int row0 = row0_wg + wave * 32;
    const int row = row0 + l32;
    const bool row_ok = row < a.R;
    const int nb = row_ok ? row / a.G : 0;           // n*B + b
    const int g = row_ok ? row % a.G : 0;
    const int my_rollout = row_ok ? nb / a.B : -1;
    const int my_b = row_ok ? nb % a.B : 0;            // position inside the block
    // rollouts spanned by this wave's rows and by the whole M-tile
    const int wave_n_lo = row0 / BG;
    const int wave_n_hi = (min(row0 + 31, a.R - 1)) / BG;
    const bool wave_has_rows = row0 < a.R;
    const int wg_n_lo = row0_wg / BG;
    const int wg_n_hi = (min(row0_wg + MROWS - 1, a.R - 1)) / BG;

    // ---- Q fragments: B operand of S^T = K Q^T ------------------------------
    // (loaded after the first K/V tiles have been requested, so the two latencies overlap)
    bf16x8 qf[KS];
    auto load_q = [&]() {
        const uint16_t* qp = a.q + ((size_t)nb * a.Hq + (size_t)kh * a.G + g) * D + half * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            u32x4 raw = {0u, 0u, 0u, 0u};
            if (row_ok) raw = *reinterpret_cast<const u32x4*>(qp + ks * 16);
            qf[ks] = __builtin_bit_cast(bf16x8, raw);
        }
    };

    // ---- tile schedule -------------------------------------------------------
    const int t0 = min(t_begin, a.TP);
    const int n_prefix = min(t_end, a.TP) - t0;
    const int tail_tiles_per_rollout = (a.B + KT - 1) / KT;
    // the segment that ends the M-tile's key range also takes the in-block tail
    const int n_tail = (t_end == a.TPU) ? (wg_n_hi - wg_n_lo + 1) * tail_tiles_per_rollout : 0;
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
            t.key0 = 0;
        } else {
            const int j = i - n_prefix;
            const int n = wg_n_lo + j / tail_tiles_per_rollout;
            const int key0 = (j % tail_tiles_per_rollout) * KT;
            const size_t off = ((size_t)n * a.B + key0) * kv_stride + (size_t)kh * D;
            t.k = a.bk + off;
            t.v = a.bv + off;
            t.valid = min(KT, a.B - key0);
            t.rollout = n;
            t.key0 = key0;
        }
        return t;
    };

    // ---- global -> register staging of one tile -----------------------------
    u32x4 kreg[C::K_PER_THREAD];
    u32x4 vreg[C::K_PER_THREAD];

    // 16-byte pieces, consecutive lanes along a row; rows beyond `valid` are zero.
    auto load_rows = [&](u32x4 (&reg)[C::K_PER_THREAD], const uint16_t* base, int valid, bool full) {
#pragma unroll
        for (int i = 0; i < C::K_PER_THREAD; ++i) {
            const int c = tid + i * C::THREADS;
            const int key = c / (D / 8);
            const int col = c % (D / 8);
            u32x4 x = {0u, 0u, 0u, 0u};
            if (full || key < valid) x = *reinterpret_cast<const u32x4*>(base + (size_t)key * kv_stride + col * 8);
            reg[i] = x;
        }
    };
    auto store_rows = [&](const u32x4 (&reg)[C::K_PER_THREAD], unsigned char* tile, int row_bytes) {
#pragma unroll
        for (int i = 0; i < C::K_PER_THREAD; ++i) {
            const int c = tid + i * C::THREADS;
            const int key = c / (D / 8);
            const int col = c % (D / 8);
            *reinterpret_cast<u32x4*>(tile + key * row_bytes + col * 16) = reg[i];
        }
    };
    auto load_k = [&](const uint16_t* kp, int valid, bool full) { load_rows(kreg, kp, valid, full); };
    auto load_v = [&](const uint16_t* vp, int valid, bool full) { load_rows(vreg, vp, valid, full); };
    auto store_k = [&](int buf) { store_rows(kreg, lds + buf * C::K_BYTES, C::KROW); };
    auto store_v = [&](int buf) { store_rows(vreg, lds + 2 * C::K_BYTES + buf * C::V_BYTES, C::VROW); };

    // V^T fragment of one P V MFMA (16-key step t4, channel block db) by two
    // transpose reads.  In a 16-lane group, lane 4j+q points at 4 channels of
    // key row j; the read returns to lane i the 4 keys of channel i.  Element
    // e of the fragment is key 16 t4 + 8 (e/4) + 4 half + e%4, the key order of
    // the probabilities in the S^T accumulator.
    const int tr_lane_off = ((half * 4 + ((lane & 15) >> 2)) * C::VROW) + (((lane >> 4) & 1) * 16 + (lane & 3) * 4) * 2;
    auto v_frag = [&](const unsigned char* vtile, int t4, int db) -> bf16x8 {
        typedef __attribute__((address_space(3))) i16x4 lds_i16x4;
        const unsigned char* p0 = vtile + tr_lane_off + (t4 * 16) * C::VROW + db * 64;
        const i16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4*)(p0));
        const i16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4*)(p0 + 8 * C::VROW));
        typedef short i16x8 __attribute__((ext_vector_type(8)));
        const i16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        return __builtin_bit_cast(bf16x8, both);
    };

    // ---- streaming-softmax state: one query row per lane --------------------
    f32x16 o[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[db][v] = 0.f;
    float m_ref = -INFINITY;   // reference value the exponentials are taken against (raw score units)
    float l_run = 0.f;         // this lane's share of the running sum

    // scores of one 32-key block: S^T[key, row] = K[key, :] . Q[row, :]
    auto qk_block = [&](const unsigned char* kl, int kb, f32x16& s) {
#pragma unroll
        for (int v = 0; v < 16; ++v) s[v] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const bf16x8 kf = *reinterpret_cast<const bf16x8*>(kl + (kb * 32 + l32) * C::KROW + ks * 32 + half * 16);
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], s, 0, 0, 0);
        }
    };
    // maximum of a row's 64 scores (both halves of the wavefront agree on it)
    auto row_max = [&](const f32x16& s0, const f32x16& s1) -> float {
        float mx = fmaxf(s0[0], s1[0]);
#pragma unroll
        for (int v = 1; v < 16; ++v) mx = fmaxf(mx, fmaxf(s0[v], s1[v]));
        return fmaxf(mx, other_half(mx));
    };
    // raise the reference when the tile maximum outgrew it by more than 2^8
    auto update_reference = [&](float mx) {
        // also true for the first tile (m_ref = -inf); never evaluates inf - inf
        const bool need = (mx > m_ref) && ((mx - m_ref) * a.c > 8.f);
        if (__any(need)) {
            const float m_new = fmaxf(m_ref, mx);
            const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
            const float alpha = fast_exp2((m_ref - m_use) * a.c);
            l_run *= alpha;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int v = 0; v < 16; ++v) o[db][v] *= alpha;
            m_ref = m_new;
        }
    };
    // probabilities of one 32-key block, rounded to bf16 as two MFMA B operands
    auto exp_block = [&](const f32x16& s, float mc, bf16x8& p0, bf16x8& p1) {
        float acc = 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const float p = fast_exp2(fmaf(s[v], a.c, -mc));
            acc += p;
            if (v < 8) p0[v] = (__bf16)p; else p1[v - 8] = (__bf16)p;
        }
        l_run += acc;
    };
    // O^T += V^T P^T for the two 16-key steps of one 32-key block
    auto pv_block = [&](const unsigned char* vtile, int kb, const bf16x8& p0, const bf16x8& p1) {
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                const bf16x8 vf = v_frag(vtile, kb * 2 + u, db);
                o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, u == 0 ? p0 : p1, o[db], 0, 0, 0);
            }
    };

    // ---- fast path: full prefix tiles, software pipelined ---------------------
    // F leading tiles of this piece are complete 64-key prefix tiles.
    const int F = (n_prefix > 0 && (t0 + n_prefix) * KT > a.L) ? n_prefix - 1 : n_prefix;
    const uint16_t* pk0 = a.pk + (size_t)t0 * KT * kv_stride + (size_t)kh * D;
    const uint16_t* pv0 = a.pv + (size_t)t0 * KT * kv_stride + (size_t)kh * D;
    const size_t tile_elems = (size_t)KT * kv_stride;
    // LDS: two K buffers then two V buffers (padded register-staged layout or unpadded direct layout)
    constexpr int KB_BYTES = PACKED ? C::T_BYTES : C::K_BYTES;
    constexpr int VB_BYTES = PACKED ? C::T_BYTES : C::V_BYTES;
    unsigned char* const kbuf0 = lds;
    unsigned char* const vbuf0 = lds + 2 * KB_BYTES;
    bf16x8 p[4];      // probabilities of a tile as MFMA B operands, one per 16-key step

    // direct path: per-lane byte offsets of the pieces this lane moves, and of
    // the fragments it reads
    typedef __attribute__((address_space(3))) void lds_void;
    __amdgpu_buffer_rsrc_t k_rsrc, v_rsrc;
    uint32_t k_voff[C::NI], v_voff[C::NI], k_fragoff[KS];
    const uint32_t v_fragoff = (uint32_t)(half * (D * 16) + l32 * 16);   // packed V^T: [16-key step][half][d][8 keys]
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);   // same value, known to be wave-uniform
    if (PACKED) {
        k_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(a.pk), 0, a.L * a.Hkv * D * 2, 0x00020000);
        v_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(a.vt), 0, a.Hkv * a.TPF * C::T_BYTES, 0x00020000);
#pragma unroll
        for (int j = 0; j < C::NI; ++j) {
            const int piece = wave * C::NI + j;
            const int r = piece * C::RPB + lane / C::CH;          // key row of this lane's 16 bytes
            const int c = (lane % C::CH) ^ ((r / C::RPL) & (C::CH - 1));   // which piece of the row lands here
            k_voff[j] = (uint32_t)(r * (int)kv_stride * 2 + c * 16);
            v_voff[j] = (uint32_t)(piece * 1024 + lane * 16);
        }
        const int y = ((l32 / C::RPL) & (C::CH - 1)) ^ half;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) k_fragoff[ks] = (uint32_t)(l32 * D * 2 + (((2 * ks) ^ y) << 4));
    }
    // start moving prefix tile `t` (index inside this segment) into buffer `buf`
    auto fetch_k = [&](int t, int buf) {
        if (PACKED) {
            const uint32_t soff = __builtin_amdgcn_readfirstlane((uint32_t)(((size_t)(t0 + t) * KT * kv_stride + (size_t)kh * D) * 2));
#pragma unroll
            for (int j = 0; j < C::NI; ++j)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(k_rsrc, (lds_void*)(kbuf0 + buf * KB_BYTES + (wave_u * C::NI + j) * 1024),
                                                         16, k_voff[j], soff, 0, 0);
        } else {
            load_k(pk0 + (size_t)t * tile_elems, KT, true);
        }
    };
    auto fetch_v = [&](int t, int buf) {
        if (PACKED) {
            const uint32_t soff = __builtin_amdgcn_readfirstlane((uint32_t)(((size_t)kh * a.TPF + (t0 + t)) * C::T_BYTES));
#pragma unroll
            for (int j = 0; j < C::NI; ++j)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(v_rsrc, (lds_void*)(vbuf0 + buf * VB_BYTES + (wave_u * C::NI + j) * 1024),
                                                         16, v_voff[j], soff, 0, 0);
        } else {
            load_v(pv0 + (size_t)t * tile_elems, KT, true);
        }
    };
    // make the fetched tiles visible to the workgroup
    auto publish = [&]() {
        if (PACKED) __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): the direct loads have landed
        __syncthreads();
    };
    // fragments of the fast path.  K: key block kb (32 keys), k-step ks.
    auto k_frag_fast = [&](int buf, int kb, int ks) -> bf16x8 {
        if (PACKED) return *reinterpret_cast<const bf16x8*>(kbuf0 + buf * KB_BYTES + kb * 32 * D * 2 + k_fragoff[ks]);
        return *reinterpret_cast<const bf16x8*>(kbuf0 + buf * KB_BYTES + (kb * 32 + l32) * C::KROW + ks * 32 + half * 16);
    };
    // V^T: 16-key step t4, channel block db
    auto v_frag_fast = [&](int buf, int t4, int db) -> bf16x8 {
        if (PACKED) return *reinterpret_cast<const bf16x8*>(vbuf0 + buf * VB_BYTES + t4 * (D * 32) + db * 512 + v_fragoff);
        return v_frag(vbuf0 + buf * VB_BYTES, t4, db);
    };

    if (F > 0) {
        // prologue: K(0), V(0) and K(1) into LDS, scores of tile 0
        fetch_k(0, 0);
        fetch_v(0, 0);
        load_q();
        if (!PACKED) {
            store_k(0);
            store_v(0);
        }
        fetch_k(min(1, F - 1), 1);
        if (!PACKED) store_k(1);
        publish();
        f32x16 sa[2], sb[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
            for (int v = 0; v < 16; ++v) sa[kb][v] = 0.f;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                sa[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k_frag_fast(0, kb, ks), qf[ks], sa[kb], 0, 0, 0);
        }
        __syncthreads();   // K buffer 0 is refilled during the first step

        // One pipelined step: probabilities and P V of tile i from s_cur while
        // the scores of tile i+1 go to s_nxt; K(i+2) and V(i+1) are fetched.
        //   slots  0- 7  S(i+1) first 32 keys   ||  row maximum of tile i
        //   slots  8-15  S(i+1) second 32 keys  ||  exp of the first 32 keys
        //   slots 16-23  P V first 32 keys      ||  exp of the second 32 keys
        //   slots 24-31  P V second 32 keys     ||  staging of the fetched tiles
        // `par` is i % 2 as a compile-time constant (buffer offsets become
        // immediates), `nxt` says whether tile i+1 exists.
        auto step = [&](auto par, auto nxt, int i, f32x16 (&s_cur)[2], f32x16 (&s_nxt)[2]) {
            constexpr int P = decltype(par)::value;
            constexpr bool has_next = decltype(nxt)::value;
            // the buffers refilled here were last read in the previous step
            fetch_k(min(i + 2, F - 1), P);
            fetch_v(min(i + 1, F - 1), 1 - P);
            auto kfrag = [&](int kb, int ks) { return k_frag_fast(1 - P, kb, ks); };
            // P V slot j of block kb: 16-key step j / DB, channel block j % DB
            auto vfrag = [&](int kb, int j) { return v_frag_fast(P, kb * 2 + j / DB, j % DB); };
            bf16x8 f[3];
            FDD_SCHED_FENCE();

            // ---- slots 0-7 ----
            float mx = -INFINITY;
            if (has_next) {
                f[0] = kfrag(0, 0);
                f[1] = kfrag(0, 1);
#pragma unroll
                for (int v = 0; v < 16; ++v) s_nxt[0][v] = 0.f;
            }
#pragma unroll
            for (int j = 0; j < KS; ++j) {
                if (has_next) {
                    if (j + 2 < KS) f[(j + 2) % 3] = kfrag(0, j + 2);
                    s_nxt[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[j % 3], qf[j], s_nxt[0], 0, 0, 0);
                }
#pragma unroll
                for (int v = j * (16 / KS); v < (j + 1) * (16 / KS); ++v) {
                    mx = fmaxf(fmaxf(mx, s_cur[0][v]), s_cur[1][v]);
                }
                FDD_PIN(mx);
                FDD_SCHED_FENCE();
            }
            mx = fmaxf(mx, other_half(mx));
            update_reference(mx);
            const float mc = ((m_ref == -INFINITY) ? 0.f : m_ref) * a.c;
            float acc = 0.f;
            u32x4 pw[4];     // the B operands of P V as packed words
            // four probabilities of block kb (registers 4e .. 4e+3), rounded into the B operands
            auto exp_quad = [&](int kb, int e) {
                float pr[4];
#pragma unroll
                for (int t = 0; t < 4; ++t) pr[t] = fast_exp2(fmaf(s_cur[kb][4 * e + t], a.c, -mc));
                acc += (pr[0] + pr[1]) + (pr[2] + pr[3]);
                typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
                bf16x2 lo = {(__bf16)pr[0], (__bf16)pr[1]}, hi = {(__bf16)pr[2], (__bf16)pr[3]};
                uint32_t ulo = __builtin_bit_cast(uint32_t, lo), uhi = __builtin_bit_cast(uint32_t, hi);
                FDD_PIN(ulo);
                FDD_PIN(uhi);
                FDD_PIN(acc);
                pw[kb * 2 + e / 2][(e & 1) * 2] = ulo;
                pw[kb * 2 + e / 2][(e & 1) * 2 + 1] = uhi;
            };
            FDD_SCHED_FENCE();

            // ---- slots 8-15 ----
            if (has_next) {
                f[0] = kfrag(1, 0);
                f[1] = kfrag(1, 1);
#pragma unroll
                for (int v = 0; v < 16; ++v) s_nxt[1][v] = 0.f;
            }
#pragma unroll
            for (int j = 0; j < KS; ++j) {
                if (has_next) {
                    if (j + 2 < KS) f[(j + 2) % 3] = kfrag(1, j + 2);
                    s_nxt[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[j % 3], qf[j], s_nxt[1], 0, 0, 0);
                }
                if ((j * 4) % KS == 0) exp_quad(0, j * 4 / KS);
                FDD_SCHED_FENCE();
            }
            p[0] = __builtin_bit_cast(bf16x8, pw[0]);
            p[1] = __builtin_bit_cast(bf16x8, pw[1]);

            // ---- slots 16-23 ----
            constexpr int PVS = 2 * DB;      // P V MFMAs per 32-key block
            f[0] = vfrag(0, 0);
            f[1] = vfrag(0, 1);
#pragma unroll
            for (int j = 0; j < PVS; ++j) {
                if (j + 2 < PVS) f[(j + 2) % 3] = vfrag(0, j + 2);
                o[j % DB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[j % 3], p[j / DB], o[j % DB], 0, 0, 0);
                if ((j * 4) % PVS == 0) exp_quad(1, j * 4 / PVS);
                FDD_SCHED_FENCE();
            }
            p[2] = __builtin_bit_cast(bf16x8, pw[2]);
            p[3] = __builtin_bit_cast(bf16x8, pw[3]);
            l_run += acc;

            // ---- slots 24-31 ----
            f[0] = vfrag(1, 0);
            f[1] = vfrag(1, 1);
#pragma unroll
            for (int j = 0; j < PVS; ++j) {
                if (j + 2 < PVS) f[(j + 2) % 3] = vfrag(1, j + 2);
                o[j % DB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[j % 3], p[2 + j / DB], o[j % DB], 0, 0, 0);
                if (!PACKED) {
                    if (j == 1) store_k(P);
                    if (j == PVS / 2 + 1) store_v(1 - P);
                }
                FDD_SCHED_FENCE();
            }
            publish();
        };
        using std::integral_constant;
        const integral_constant<int, 0> even;
        const integral_constant<int, 1> odd;
        const integral_constant<bool, true> more;
        const integral_constant<bool, false> last;
        int i = 0;
        for (; i + 2 < F; i += 2) {
            step(even, more, i, sa, sb);
            step(odd, more, i + 1, sb, sa);
        }
        if (i + 2 == F) {
            step(even, more, i, sa, sb);
            step(odd, last, i + 1, sb, sa);
        } else {
            step(even, last, i, sa, sb);
        }
    } else {
        load_q();
    }
    f32x16 s[2];      // scores of a masked tile

    // ---- masked path: ragged last prefix tile and the in-block tail ------------
    for (int i = F; i < n_tiles; ++i) {
        const Tile t = tile_at(i);
        load_k(t.k, t.valid, false);
        load_v(t.v, t.valid, false);
        store_rows(kreg, lds, C::KROW);
        store_rows(vreg, lds + C::K_BYTES, C::VROW);
        __syncthreads();
        const bool wave_active = wave_has_rows &&
            (t.rollout < 0 || (t.rollout >= wave_n_lo && t.rollout <= wave_n_hi));
        if (wave_active) {
            qk_block(lds, 0, s[0]);
            qk_block(lds, 1, s[1]);
            // register v of block kb is key kb*32 + (v/4)*8 + half*4 + v%4
            const bool row_sees = (t.rollout < 0) || (t.rollout == my_rollout);
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int key = kb * 32 + (v >> 2) * 8 + half * 4 + (v & 3);
                    const bool later = a.causal && t.rollout >= 0 && t.key0 + key > my_b;   // verify pass: causal inside the block
                    if (!row_sees || key >= t.valid || later) s[kb][v] = -INFINITY;
                }
            update_reference(row_max(s[0], s[1]));
            const float mc = ((m_ref == -INFINITY) ? 0.f : m_ref) * a.c;
            exp_block(s[0], mc, p[0], p[1]);
            exp_block(s[1], mc, p[2], p[3]);
            pv_block(lds + C::K_BYTES, 0, p[0], p[1]);
            pv_block(lds + C::K_BYTES, 1, p[2], p[3]);
        }
        __syncthreads();
    }
    const float m_run = m_ref;

    // ---- epilogue of the segment ------------------------------------------------
    const float l_tot = l_run + other_half(l_run);
    if (row_ok) {
        if (n_seg == 1) {
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
            const size_t prow = ((size_t)M * a.max_seg + seg) * MROWS + (wave * 32 + l32);
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
    }   // next segment of this workgroup's range
#endif
}

// ---------------------------------------------------------------------------
// Pre-pass: the full 64-key prefix tiles of V, repacked once into the order
// the P V fragments are read in:  vt[kh][tile][t4][half][d][8 keys], where the
// 8 keys of (t4, half) are 16 t4 + 4 half + {0..3} and 16 t4 + 8 + 4 half + {0..3}
// (the key order of the probabilities in the S^T accumulator).  One workgroup
// per (tile, KV head): stage the tile [key][d] in LDS, then let the LDS
// transpose read do the transposition; a wavefront stores two 512-byte runs.
template <int D>
__global__ __launch_bounds__(512) void vt_pack_kernel(const uint16_t* __restrict__ pv, uint16_t* __restrict__ vt,
                                                       int Hkv, int TPF)
{
    using C = Cfg<D, 8>;
    constexpr int DB = D / 32;
    __shared__ __align__(16) unsigned char tile[C::V_BYTES];
    const int t = blockIdx.x, kh = blockIdx.y;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, half = lane >> 5;
    const size_t kv_stride = (size_t)Hkv * D;
    const uint16_t* src = pv + (size_t)t * KT * kv_stride + (size_t)kh * D;
#pragma unroll
    for (int i = 0; i < C::K_PER_THREAD; ++i) {
        const int c = tid + i * C::THREADS;
        const int key = c / (D / 8), col = c % (D / 8);
        *reinterpret_cast<u32x4*>(tile + key * C::VROW + col * 16) =
            *reinterpret_cast<const u32x4*>(src + (size_t)key * kv_stride + col * 8);
    }
    __syncthreads();
    const int tr_lane_off = ((half * 4 + ((lane & 15) >> 2)) * C::VROW) + (((lane >> 4) & 1) * 16 + (lane & 3) * 4) * 2;
    unsigned char* dst = reinterpret_cast<unsigned char*>(vt) + ((size_t)kh * TPF + t) * C::T_BYTES;
    for (int combo = wave; combo < 4 * DB; combo += 8) {
        const int t4 = combo / DB, db = combo % DB;
        typedef __attribute__((address_space(3))) i16x4 lds_i16x4;
        const unsigned char* p0 = tile + tr_lane_off + (t4 * 16) * C::VROW + db * 64;
        const i16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4*)(p0));
        const i16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4*)(p0 + 8 * C::VROW));
        typedef short i16x8 __attribute__((ext_vector_type(8)));
        const i16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        *reinterpret_cast<i16x8*>(dst + t4 * (D * 32) + half * (D * 16) + (db * 32 + l32) * 16) = both;
    }
}

template <int D, int WAVES, bool PACKED>
hipError_t launch(const Args& a, bool pack_now, hipStream_t stream, hipEvent_t before_main)
{
    using C = Cfg<D, WAVES>;
    const size_t lds_bytes = PACKED ? 4 * (size_t)C::T_BYTES : 2 * (size_t)C::BUF_BYTES;
    static_assert(4 * C::T_BYTES >= C::BUF_BYTES, "the masked path stages one padded K and V tile");
    const auto kern = &attn_bf16_kernel<D, WAVES, PACKED>;
    static bool attr_done = false;   // per instantiation
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    if (PACKED && pack_now) {
        hipLaunchKernelGGL(vt_pack_kernel<D>, dim3(a.TPF, a.Hkv), dim3(512), 0, stream, a.pv, const_cast<uint16_t*>(a.vt),
                           a.Hkv, a.TPF);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (before_main) {
        hipError_t e = hipEventRecord(before_main, stream);
        if (e != hipSuccess) return e;
    }
    const int grid = (a.W + kNumXCD - 1) / kNumXCD * kNumXCD;   // padded so that every XCD gets the same count
    hipLaunchKernelGGL(kern, dim3(grid), dim3(C::THREADS), lds_bytes, stream, a);
    return hipGetLastError();
}

}  // namespace attn_bf16

using namespace attn_bf16;

hipError_t launch_attn_bf16(const fdd_attn_params& p, const AttnPlan& plan, float scale, hipStream_t s, hipEvent_t before_main)
{
    Args a;
    a.q = static_cast<const uint16_t*>(p.q);
    a.pk = static_cast<const uint16_t*>(p.prefix_k);
    a.pv = static_cast<const uint16_t*>(p.prefix_v);
    a.bk = static_cast<const uint16_t*>(p.block_k);
    a.bv = static_cast<const uint16_t*>(p.block_v);
    a.out = static_cast<uint16_t*>(p.out);
    char* ws = static_cast<char*>(p.workspace);
    a.ws_o = reinterpret_cast<float*>(ws);
    a.ws_ml = reinterpret_cast<float*>(ws + plan.ws_o_bytes);
    const bool pack_now = plan.packed && !p.prefix_v_packed;
    a.vt = pack_now ? reinterpret_cast<const uint16_t*>(ws + plan.ws_o_bytes + plan.ws_ml_bytes)
                    : static_cast<const uint16_t*>(p.prefix_v_packed);
    a.N = p.N; a.B = p.B; a.L = p.L; a.Hq = p.Hq; a.Hkv = p.Hkv;
    a.G = plan.G; a.R = plan.R; a.MT = plan.MT; a.TP = plan.TP; a.TPF = p.L / 64;
    a.TPU = plan.TPU; a.W = plan.W; a.max_seg = plan.max_seg; a.U = plan.U; a.S = plan.uniform;
    a.causal = (p.flags & FDD_ATTN_CAUSAL_BLOCK) ? 1 : 0;
    a.c = scale * 1.4426950408889634f;
    if (plan.mtile_rows != 256) return hipErrorInvalidValue;
    if (plan.packed)
        return p.D == 128 ? launch<128, 8, true>(a, pack_now, s, before_main) : launch<64, 8, true>(a, pack_now, s, before_main);
    return p.D == 128 ? launch<128, 8, false>(a, false, s, before_main) : launch<64, 8, false>(a, false, s, before_main);
}

hipError_t launch_prefix_pack(const void* prefix_v, int L, int Hkv, int D, void* packed, hipStream_t s)
{
    const int TPF = L / KT;
    if (TPF == 0) return hipSuccess;
    const uint16_t* src = static_cast<const uint16_t*>(prefix_v);
    uint16_t* dst = static_cast<uint16_t*>(packed);
    if (D == 128) hipLaunchKernelGGL(vt_pack_kernel<128>, dim3(TPF, Hkv), dim3(512), 0, s, src, dst, Hkv, TPF);
    else hipLaunchKernelGGL(vt_pack_kernel<64>, dim3(TPF, Hkv), dim3(512), 0, s, src, dst, Hkv, TPF);
    return hipGetLastError();
}

}  // namespace fdd
