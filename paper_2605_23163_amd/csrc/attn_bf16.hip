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
//   * Every K/V tile goes from global memory straight into LDS
//     (buffer_load ... lds: no registers, no vector ALU work, no LDS writes by
//     the waves) into a ring of 4 K slots and 4 V slots.  K tiles lie
//     [key][d] with the 16-byte pieces of a row XOR-swizzled by the row index,
//     which keeps the K fragment reads conflict-free without padding.
//   * O^T += V^T P^T needs, per lane, 8 keys of one channel, i.e. V with the
//     key index contiguous, while V lies in memory [key][d].  Where an
//     M-tile's keys are streamed by more than one workgroup (R > 256 rows per
//     KV head), or the caller did it once for the prefix, the full prefix
//     tiles of V are packed into the exact fragment order,
//     [tile][16-key step][half][d][8 keys], and read back as plain
//     conflict-free 128-bit loads.  V tiles that are moved as they lie (a
//     single M-tile per head, the ragged last prefix tile, a rollout's private
//     tiles) are read with the gfx950 LDS transpose read (ds_read_b64_tr_b16:
//     lane i of a 16-lane group receives column i of a 4 x 16 block, i.e. 4
//     consecutive keys of channel i); their 32-byte columns are XOR-swizzled
//     by the row on the global side of the load, which makes those reads
//     conflict-free too.
//   * Full prefix tiles run through a software-pipelined loop written as 32
//     slots per tile, one per MFMA.  Each slot also carries a slice of vector
//     ALU work that does not depend on that MFMA: while the matrix pipe
//     produces the scores of tile i+1 and then the P V products of tile i,
//     the vector ALUs reduce the row maximum of tile i, take its exponentials
//     and round them to bf16.  One wavefront can only issue a vector
//     instruction every other issue slot, so two wavefronts per SIMD running
//     this same mix are what fills both pipes.  V of tile i+3 and K of tile
//     i+4 are requested at the start of step i (K is read one step before V,
//     so its slot is free one step earlier) and waits are counted (the loads
//     of a wavefront complete in issue order), so four half tiles stay in
//     flight across a step boundary; LDS
//     fragments are requested two MFMAs before their use.  The loop is
//     unrolled four times so that ring slots are immediate offsets.
//   * The softmax reference value of a row is only raised when the running
//     maximum outgrows it by more than 2^8; in between probabilities may
//     exceed 1, which fp32 sums and bf16 relative precision do not mind, and
//     the accumulator rescale becomes a rare wave-uniform branch.  The result
//     is mathematically the same softmax.
//   * Work is dealt out in units of one 64-key prefix tile of one M-tile.
//     Either every M-tile is cut into S equal pieces (workgroups numbered so
//     that an XCD owns all M-tiles of one (KV head, piece): they walk the same
//     keys in step and the XCD's L2 serves all but the first fetch), or all
//     units, ordered by (KV head, M-tile, tile), are cut into W contiguous
//     ranges, one per workgroup (stream-K), so every compute unit gets the
//     same amount of work whatever the shape.  A range may end inside an
//     M-tile and continue in the next one: each such segment keeps its own
//     streaming-softmax state (m, l, o) per row.  An M-tile that was covered
//     by a single segment is normalised and written as bf16 output directly;
//     otherwise the segments leave fp32 partials that a second small kernel
//     merges (log-sum-exp merge, fixed order).
//   * The ragged last prefix tile and the private tiles of every rollout the
//     M-tile's rows belong to (the rows that rollout committed since the fork,
//     then its live block: paper, "Shared prefix" and "Block-Causal
//     Diffusion") go through a simpler masked path out of the same ring: rows
//     of other rollouts are masked to -inf, and in the verify pass of scaffold
//     speculative decoding the block keys after the query's own position too.
#include <atomic>
#include <type_traits>

#include "fdd_internal.h"

namespace fdd {
namespace attn_bf16 {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;
typedef __attribute__((__vector_size__(2 * sizeof(uint32_t)))) uint32_t u32x2;

constexpr int ODD_XCD_WEIGHT = 97;   // share of a piece on an odd XCD, in per cent of one on an even XCD (measured: 96..98 alike)
constexpr int KT = 64;           // keys per tile
constexpr int NB = 4;            // ring slots per operand in LDS
typedef short i16x4 __attribute__((ext_vector_type(4)));

// Kernel arguments.  They are read from memory with scalar loads, a 64-byte line at a time, and every
// first touch of a line is a round trip of a few hundred nanoseconds: the fields a workgroup needs before
// it can request its first tiles come first and are pulled in together (see the top of the kernel), the
// fields of the Q load follow, the rest is only needed while the first tiles are on their way.
struct Args {
    // ---- before the first tile request -----------------------------------------------------------
    const uint16_t* pk;
    const uint16_t* pv;
    const uint16_t* vt;   // packed V^T tiles of the full prefix tiles (PACKED kernels only)
    long long p_bs, vt_bs;   // batch: element strides between the problems' prefix arrays
    int W;          // workgroups
    int per_xcd;    // ceil(W / 8)
    int S;          // > 0: every M-tile is cut into S equal pieces (W = Hkv*MT*S); 0: free ranges
    int MT, TPU;    // M-tiles per KV head; units per M-tile = max(TP, 1) + booked private units
    int base, rem;  // free ranges: U / W and U % W
    int w_even, w_odd;   // equal pieces: weight of a piece by the parity of the XCD it runs on
    int Hkv, batch;      // batch: independent problems in this launch
    int L, TP, TPF;      // prefix rows, prefix tiles, full prefix tiles = L / 64
    FastDiv dMT, dS, dTPU, dHkv, dPerXcd;   // divisions by launch constants
    // ---- the Q load ----------------------------------------------------------------------------------
    const uint16_t* q;
    const int32_t* qpos;   // stacked rows are the listed block positions only (ascending n*B + b), or nullptr: all of them
    long long q_bs;
    int G, R, Hq, NB;      // NB = N * B
    FastDiv dG;
    // ---- the rest ------------------------------------------------------------------------------------
    const uint16_t* bk;
    const uint16_t* bv;
    const uint16_t* ek;   // per-rollout extension [N, Ecap, Hkv, D]
    const uint16_t* ev;
    uint16_t* out;
    void* ws_o;      // partial averages, bf16, in accumulator order (see the epilogue)
    float* ws_ml;    // partial (m, l) per row
    long long b_bs, e_bs, o_bs;
    int E, Ecap;
    int N, B;
    int max_seg;    // partial slots per M-tile
    int causal;     // in-block keys are visible up to the query's own position only
    float c;        // scale * log2(e)
    int ttpr;       // private tiles per rollout: extension tiles, then block tiles
    FastDiv dB, dBG, dTTPR, dBase, dBase1;
};

template <int D, int WAVES>
struct Cfg {
    static constexpr int THREADS = WAVES * 64;
    // 64 x D tiles, unpadded, moved global -> LDS in 1 KB pieces, one per wavefront instruction
    static constexpr int T_BYTES = KT * D * 2;
    static constexpr int NI = T_BYTES / 1024 / WAVES;    // pieces per wavefront and tile
    static constexpr int IPT = 2 * NI;                   // load instructions per wavefront for K and V of one tile
    static constexpr int CH = D / 8;                     // 16-byte pieces per row
    static constexpr int RPB = 1024 / (D * 2);           // rows per 1 KB piece
    static constexpr int RPL = 256 / (D * 2);            // rows per 256-byte bank line
    static constexpr int V_RING = NB * T_BYTES;          // LDS offset of the V ring (the K ring starts at 0)
    static constexpr int LDS_BYTES = 2 * NB * T_BYTES;
    static_assert(NI >= 1 && T_BYTES % (1024 * WAVES) == 0, "tile must divide over the wavefronts");
    static_assert(3 * IPT < 64, "outstanding loads must fit the counter");
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

// Wait until at most N of this wavefront's vector memory operations are
// still in flight (they complete in issue order).
template <int N>
__device__ __forceinline__ void wait_vm()
{
    static_assert(N >= 0 && N < 64, "counter range");
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

// Workgroup barrier that orders LDS traffic only.  (__syncthreads() also
// fences global memory, which makes the compiler drain every tile still on
// its way into the ring.)  No memory access is moved across it.
__device__ __forceinline__ void wg_barrier() { asm volatile("s_barrier" ::: "memory"); }

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
    constexpr uint32_t RSRC_FLAGS = 0x00020000;

    extern __shared__ __align__(16) unsigned char lds[];
    typedef __attribute__((address_space(3))) void lds_void;

    const int tid = threadIdx.x;
    const int wave = tid >> 6;
    const int lane = tid & 63;
    const int l32 = lane & 31;
    const int half = lane >> 5;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);   // same value, known to be wave-uniform

    // ---- everything the first tile requests need, in one round trip to the argument block -------
    {
        long long h0 = a.p_bs, h1 = a.vt_bs;
        int h2 = a.W, h3 = a.per_xcd, h4 = a.S, h5 = a.MT, h6 = a.TPU, h7 = a.base, h8 = a.rem, h9 = a.w_even,
            h10 = a.w_odd, h11 = a.Hkv, h12 = a.batch, h13 = a.L, h14 = a.TP, h15 = a.TPF;
        uint32_t d0 = a.dMT.mul, d1 = a.dMT.shift, d2 = a.dS.mul, d3 = a.dS.shift, d4 = a.dTPU.mul, d5 = a.dTPU.shift,
                 d6 = a.dHkv.mul, d7 = a.dHkv.shift, d8 = a.dPerXcd.mul, d9 = a.dPerXcd.shift;
        const uint16_t *p0 = a.pk, *p1 = a.pv, *p2 = a.vt;
        asm volatile("" ::"s"(h0), "s"(h1), "s"(h2), "s"(h3), "s"(h4), "s"(h5), "s"(h6), "s"(h7), "s"(h8), "s"(h9), "s"(h10),
                     "s"(h11), "s"(h12), "s"(h13), "s"(h14), "s"(h15), "s"(d0), "s"(d1), "s"(d2), "s"(d3), "s"(d4), "s"(d5),
                     "s"(d6), "s"(d7), "s"(d8), "s"(d9), "s"(p0), "s"(p1), "s"(p2));
        // the fields of the Q load, and a first touch of every other 64-byte line of the block (what is read
        // from those later then comes from the scalar cache)
        const uint16_t* q0 = a.q;
        const int32_t* q1 = a.qpos;
        long long q2 = a.q_bs;
        int q3 = a.G, q4 = a.R, q5 = a.Hq, q6 = a.NB;
        uint32_t q7 = a.dG.mul, q8 = a.dG.shift;
        const uint32_t* ap = reinterpret_cast<const uint32_t*>(&a);
        static_assert(sizeof(Args) > 80 * 4 && sizeof(Args) <= 96 * 4, "one touch per 64-byte line of Args");
        uint32_t t3 = ap[48], t4 = ap[64], t5 = ap[80];
        asm volatile("" ::"s"(q0), "s"(q1), "s"(q2), "s"(q3), "s"(q4), "s"(q5), "s"(q6), "s"(q7), "s"(q8), "s"(t3), "s"(t4), "s"(t5));
    }

    // ---- this workgroup's share of the (M-tile, prefix tile) units ------------
    // Workgroups are dealt to the 8 XCDs round-robin by their launch index;
    // ranges are numbered so that the workgroups of one XCD own neighbours.
    int wg = (int)(blockIdx.x % kNumXCD) * a.per_xcd + (int)(blockIdx.x / kNumXCD);
    if (wg >= a.W) return;
    int M, t_begin, todo, piece = 0;
    if (a.S > 0) {
        // equal pieces: neighbours are the M-tiles of one (KV head, piece), which
        // walk the same keys in step, so each XCD fetches its share of K/V once
        const int rest = fast_div(wg, a.dMT), mt_ = wg - rest * a.MT;
        const int khv_ = fast_div(rest, a.dS);
        piece = rest - khv_ * a.S;
        M = khv_ * a.MT + mt_;
        if (a.w_odd == a.w_even) {
            t_begin = fast_div(a.TPU * piece, a.dS);
            todo = fast_div(a.TPU * (piece + 1), a.dS) - t_begin;
        } else {
            // The share of a piece follows the speed of the XCD it runs on (measured: the odd XCD of a
            // pair streams the same tiles a few per cent slower).  Every piece of the M-tile works out
            // the same boundaries: unit TPU * (weights before it) / (all weights).
            int cum = 0, lo = 0, hi = 0;
            for (int p = 0; p < a.S; ++p) {
                const int x = fast_div((khv_ * a.S + p) * a.MT + mt_, a.dPerXcd);
                const int wgt = (x & 1) ? a.w_odd : a.w_even;
                lo = p == piece ? cum : lo;
                cum += wgt;
                hi = p == piece ? cum : hi;
            }
            t_begin = (a.TPU * lo) / cum;
            todo = (a.TPU * hi) / cum - t_begin;
        }
    } else {
        const int u0 = unit_begin(wg, a.base, a.rem);
        todo = unit_begin(wg + 1, a.base, a.rem) - u0;
        M = fast_div(u0, a.dTPU);
        t_begin = u0 - M * a.TPU;
    }

    // ---- per-lane constants of the tile movement and of the fragment reads ------
    const uint32_t stride2 = (uint32_t)(a.Hkv * D * 2);       // bytes between consecutive keys
    // K fragment of k-step ks: row l32 of a 32-key block, 16-byte piece (2 ks + half)
    // at its swizzled place, which is the place of k-step 0 with ks XORed in
    const uint32_t k_fragoff0 = (uint32_t)(l32 * D * 2 + ((((l32 / C::RPL) & (C::CH - 1)) ^ half) << 4));
    uint32_t k_fragoff[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) k_fragoff[ks] = k_fragoff0 ^ (uint32_t)(ks << 5);
    // packed V^T: [16-key step][half][d][8 keys]; the ring's offset is part of the register
    // because the offset field of an LDS read ends at 64 KB
    uint32_t v_fragoff_ring = (uint32_t)(C::V_RING + half * (D * 16) + l32 * 16);
    FDD_PIN(v_fragoff_ring);
    // Unpacked V, transposing reads.  In a 16-lane group, lane 4j+q points at 4
    // channels of key row j; the read returns to lane i the 4 keys of channel i.
    // Element e of the assembled fragment is key 16 t4 + 8 (e/4) + 4 half + e%4,
    // the key order of the probabilities in the S^T accumulator.  Channel block
    // db sits at the swizzled place of block 0 with db XORed in.
    uint32_t vtr_off0;
    {
        const int row_l = half * 4 + ((lane & 15) >> 2);
        const int x = ((lane >> 4) & 1) * 2 + ((lane & 3) >> 1);
        const int sw = (((row_l / C::RPL) & 3) << 2) & (C::CH - 1);
        vtr_off0 = (uint32_t)(row_l * D * 2 + ((x ^ sw) << 4) + (lane & 1) * 8);
    }
    uint32_t vtr_off_ring = C::V_RING + vtr_off0;
    FDD_PIN(vtr_off_ring);
    // Tile movement: piece jn of this wavefront covers rows (wave NI + jn) RPB .. of
    // a tile; this lane moves the 16 bytes that land at LDS piece (lane % CH) of
    // its row.  K: the pieces of a row are XOR-swizzled by the row's bank line.
    // V as it lies in memory: 32-byte columns are XOR-swizzled by the row, for
    // the transposing reads.  Packed V^T tiles are copied as they are.
    uint32_t k_voff[C::NI];
#pragma unroll
    for (int jn = 0; jn < C::NI; ++jn) {
        const int r = (wave * C::NI + jn) * C::RPB + lane / C::CH;
        k_voff[jn] = (uint32_t)r * stride2 + (uint32_t)(((lane % C::CH) ^ ((r / C::RPL) & (C::CH - 1))) * 16);
    }
    const uint32_t vp_voff = (uint32_t)(wave * C::NI * 1024 + lane * 16);
    auto k_frag = [&](uint32_t kbase, int kb, int ks) -> bf16x8 {
        return *reinterpret_cast<const bf16x8*>(lds + (kbase + k_fragoff[ks]) + kb * 32 * D * 2);
    };
    // `vaddr` = slot base + vtr_off0
    auto v_frag_tr_at = [&](uint32_t vaddr, int t4, int db) -> bf16x8 {
        typedef __attribute__((address_space(3))) i16x4 lds_i16x4;
        const unsigned char* p0 = lds + (vaddr ^ (uint32_t)(db << 6)) + t4 * 16 * (D * 2);
        const i16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4*)(p0));
        const i16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4*)(p0 + 8 * (D * 2)));
        typedef short i16x8 __attribute__((ext_vector_type(8)));
        const i16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        return __builtin_bit_cast(bf16x8, both);
    };

    // (wave-uniform values are marked as such, so that addresses built from them stay in scalar registers)
    M = __builtin_amdgcn_readfirstlane(M);
    t_begin = __builtin_amdgcn_readfirstlane(t_begin);
    todo = __builtin_amdgcn_readfirstlane(todo);
    for (; todo > 0; ++M, t_begin = 0) {
        const int t_end = min(a.TPU, t_begin + todo);
        todo -= t_end - t_begin;
        // M runs over (problem of the batch, KV head, M-tile)
        const int khv = fast_div(M, a.dMT);
        const int mt = M - khv * a.MT;
        const int pb = a.batch > 1 ? fast_div(khv, a.dHkv) : 0;
        const int kh = khv - pb * a.Hkv;
        // (the arrays of problem pb are addressed where they are used: few of these pointers are live at a time)
        const __amdgpu_buffer_rsrc_t pk_rsrc = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint16_t*>(a.pk + pb * a.p_bs), 0, (uint32_t)a.L * stride2, RSRC_FLAGS);
        const __amdgpu_buffer_rsrc_t pv_rsrc = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint16_t*>((PACKED ? a.vt + pb * a.vt_bs : a.pv + pb * a.p_bs)), 0,
            PACKED ? (uint32_t)(a.Hkv * a.TPF) * C::T_BYTES : (uint32_t)a.L * stride2, RSRC_FLAGS);
        // stores of the previous segment are out of the way of the load counting below
        wait_vm<0>();

        // ---- tile schedule ---------------------------------------------------
        // Tiles 0 .. F-1 are full 64-key prefix tiles; the rest are masked: the
        // ragged last prefix tile, then, if this segment ends the M-tile's key
        // range, the in-block tail of every rollout the M-tile's rows belong to.
        const int t0 = min(t_begin, a.TP);
        const int n_prefix = min(t_end, a.TP) - t0;
        const int F = (n_prefix > 0 && (t0 + n_prefix) * KT > a.L) ? n_prefix - 1 : n_prefix;

        // ---- tile j: global memory -> ring slot j % NB, no registers in between ----
        int issued = 0;
        // full prefix tile (j < F): offsets were prepared once, only the scalar tile offset changes
        auto fetch_k = [&](int j, uint32_t slot) {        // slot = (j % NB) * T_BYTES, a constant where it matters
            const uint32_t soff = (uint32_t)((t0 + j) * KT) * stride2 + (uint32_t)(kh * D * 2);
            unsigned char* const kdst = lds + slot + wave_u * (C::NI * 1024);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(pk_rsrc, (lds_void*)kdst, 16, k_voff[0], soff, 0, 0);
            if (C::NI > 1) __builtin_amdgcn_raw_ptr_buffer_load_lds(pk_rsrc, (lds_void*)(kdst + 1024), 16, k_voff[C::NI - 1], soff, 0, 0);
        };
        auto fetch_v = [&](int j, uint32_t slot) {
            unsigned char* const vdst = lds + slot + wave_u * (C::NI * 1024) + C::V_RING;
            if (PACKED) {
                const uint32_t voff = (uint32_t)(kh * a.TPF + t0 + j) * C::T_BYTES;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(pv_rsrc, (lds_void*)vdst, 16, vp_voff, voff, 0, 0);
                if (C::NI > 1) __builtin_amdgcn_raw_ptr_buffer_load_lds(pv_rsrc, (lds_void*)(vdst + 1024), 16, vp_voff + 1024, voff, 0, 0);
            } else {
                const uint32_t soff = (uint32_t)((t0 + j) * KT) * stride2 + (uint32_t)(kh * D * 2);
                int tid_f = tid;
                FDD_PIN(tid_f);     // recomputed at every fetch rather than kept in registers
#pragma unroll
                for (int jn = 0; jn < C::NI; ++jn) {
                    const int r = ((tid_f >> 6) * C::NI + jn) * C::RPB + (tid_f & 63) / C::CH;
                    const uint32_t col16 = (uint32_t)((((tid_f & 63) % C::CH) ^ ((((r / C::RPL) & 3) << 2) & (C::CH - 1))) * 16);
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(pv_rsrc, (lds_void*)(vdst + jn * 1024), 16,
                                                             (uint32_t)r * stride2 + col16, soff, 0, 0);
                }
            }
        };
        auto fetch_full = [&](int j, uint32_t slot) {
            fetch_k(j, slot);
            fetch_v(j, slot);
        };
        // ---- Q fragments: B operand of S^T = K Q^T ------------------------------
        const int row0_wg = mt * MROWS;
        const int row0 = row0_wg + wave * 32;
        const int row = row0 + l32;
        const bool row_ok = row < a.R;
        // a stacked row is (entry of the list of query positions, query head of the group)
        const int sel = row_ok ? fast_div(row, a.dG) : 0;
        const int g = row_ok ? row - sel * a.G : 0;
        const int nb = a.qpos ? min(max(a.qpos[sel], 0), a.NB - 1) : sel;   // n*B + b
        bf16x8 qf[KS];
        {
            const uint16_t* qp = a.q + pb * a.q_bs + ((size_t)nb * a.Hq + (size_t)kh * a.G + g) * D + half * 8;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                u32x4 raw = {0u, 0u, 0u, 0u};
                if (row_ok) raw = *reinterpret_cast<const u32x4*>(qp + ks * 16);
                qf[ks] = __builtin_bit_cast(bf16x8, raw);
            }
        }
        FDD_SCHED_FENCE();

        // Q is requested first and the first full tiles right after it, before anything else is worked
        // out, so that the rest of the set-up runs under their latency.  The loads of a wavefront complete
        // in issue order: with Q in front, the first step can start as soon as Q and the first tiles are
        // there, while the later ones are still on their way.
        // (K runs one tile ahead of V: K of tile j is read one step before V of tile j, so its slot is free
        // one step earlier, and one more half tile per workgroup is on its way at any time)
        // The seven requests are issued without a branch, whatever F is: a segment with fewer than four full
        // tiles requests its last full tile again (same addresses, served by the caches; a segment with none
        // requests the last full tile of the prefix, and a prefix shorter than a tile is cut off by the buffer bounds),
        // into slots whose later contents arrive later.  Only so does the compiler know that these requests
        // follow the Q loads on every path and lets the wait for Q pass while they are in flight.
        {
            const int jmax = max(F - 1, 0);
            const int jcap = max(a.TPF - 1, 0) - t0;     // keeps t0 + j inside the full tiles (it may be negative)
#pragma unroll
            for (int j = 0; j < NB - 1; ++j) fetch_full(min(min(j, jmax), jcap), (uint32_t)j * C::T_BYTES);
            fetch_k(min(min(NB - 1, jmax), jcap), (uint32_t)(NB - 1) * C::T_BYTES);
        }
        issued = min(NB - 1, F);
        FDD_SCHED_FENCE();

        // ---- the rest of the set-up ------------------------------------------------
        int n_seg, seg;
        if (a.S > 0) {
            n_seg = a.S;
            seg = piece;
        } else {
            // owner of a unit: the first `rem` workgroups hold base + 1 units each, the others base
            const int cut = a.rem * (a.base + 1);
            auto owner = [&](int u) { return u < cut ? fast_div(u, a.dBase1) : a.rem + fast_div(u - cut, a.dBase); };
            const int first = owner(M * a.TPU);
            n_seg = owner((M + 1) * a.TPU - 1) - first + 1;
            seg = wg - first;
        }
        const int my_rollout = row_ok ? fast_div(nb, a.dB) : -1;
        const int my_b = row_ok ? nb - my_rollout * a.B : 0;   // position inside the block
        // rollouts spanned by this wave's rows and by the whole M-tile
        // (rows are in ascending order of position, hence of rollout; `r` is clamped to the rows that exist)
        auto rollout_of_row = [&](int r) {
            r = min(r, a.R - 1);
            if (!a.qpos) return fast_div(r, a.dBG);
            const int e = __builtin_amdgcn_readfirstlane(fast_div(r, a.dG));
            return fast_div(min(max(a.qpos[e], 0), a.NB - 1), a.dB);
        };
        const int wave_n_lo = rollout_of_row(row0);
        const int wave_n_hi = rollout_of_row(row0 + 31);
        const bool wave_has_rows = row0 < a.R;
        const int wg_n_lo = __builtin_amdgcn_readfirstlane(rollout_of_row(row0_wg));
        const int wg_n_hi = __builtin_amdgcn_readfirstlane(rollout_of_row(row0_wg + MROWS - 1));
        const int tte = (a.E + KT - 1) >> 6;             // tiles of a rollout's extension
        const int ttpr = a.ttpr;                         // private tiles per rollout: extension, then block
        const int n_tail = (t_end == a.TPU) ? (wg_n_hi - wg_n_lo + 1) * ttpr : 0;
        const int n_tiles = n_prefix + n_tail;

        struct Tile {
            int src;        // 0: shared prefix, 1: a rollout's extension, 2: a rollout's block
            int row_base;   // first key, as a row of that K/V array
            int valid;      // keys that exist
            int rollout;    // whose rows may see it (-1: every row)
            int key0;       // block position of the first key (block tiles)
        };
        auto tile_at = [&](int j) -> Tile {
            Tile t;
            if (j < n_prefix) {
                t.src = 0;
                t.row_base = (t0 + j) * KT;
                t.valid = min(KT, a.L - t.row_base);
                t.rollout = -1;
                t.key0 = 0;
            } else {
                const int jj = j - n_prefix;
                int n = wg_n_lo + jj, w = 0;
                if (ttpr > 1) {
                    const int q_ = fast_div(jj, a.dTTPR);
                    n = wg_n_lo + q_;
                    w = jj - q_ * ttpr;
                }
                t.rollout = n;
                if (w < tte) {
                    t.src = 1;
                    t.row_base = n * a.Ecap + w * KT;
                    t.valid = min(KT, a.E - w * KT);
                    t.key0 = 0;
                } else {
                    const int k0 = (w - tte) * KT;
                    t.src = 2;
                    t.row_base = n * a.B + k0;
                    t.valid = min(KT, a.B - k0);
                    t.key0 = k0;
                }
            }
            return t;
        };

        // masked tile: rows beyond `valid` repeat the last valid row (finite values;
        // their scores are masked), so nothing is read out of bounds
        auto fetch_masked = [&](int j) {
            const Tile t = tile_at(j);
            const uint32_t rows_in_array = t.src == 0 ? (uint32_t)a.L : t.src == 1 ? (uint32_t)(a.N * a.Ecap) : (uint32_t)(a.N * a.B);
            const uint32_t bytes = rows_in_array * stride2;
            const uint16_t* const ksrc = t.src == 0 ? a.pk + pb * a.p_bs : t.src == 1 ? a.ek + pb * a.e_bs : a.bk + pb * a.b_bs;
            const uint16_t* const vsrc = t.src == 0 ? a.pv + pb * a.p_bs : t.src == 1 ? a.ev + pb * a.e_bs : a.bv + pb * a.b_bs;
            const __amdgpu_buffer_rsrc_t k_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(ksrc), 0, bytes, RSRC_FLAGS);
            const __amdgpu_buffer_rsrc_t v_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(vsrc), 0, bytes, RSRC_FLAGS);
            const uint32_t soff = __builtin_amdgcn_readfirstlane((uint32_t)t.row_base * stride2 + (uint32_t)(kh * D * 2));
            const uint32_t slot = (uint32_t)(j & (NB - 1)) * C::T_BYTES;
            const int last = t.valid - 1;
            int tid_f = tid;
            FDD_PIN(tid_f);
            const int wave_f = tid_f >> 6, lane_f = tid_f & 63;
#pragma unroll
            for (int jn = 0; jn < C::NI; ++jn) {
                // this lane moves the 16 bytes that land at LDS piece (lane % CH) of row r of the tile
                const int r = (wave_f * C::NI + jn) * C::RPB + lane_f / C::CH;
                const uint32_t row_off = (uint32_t)min(r, last) * stride2;
                const uint32_t k_col16 = (uint32_t)(((lane_f % C::CH) ^ ((r / C::RPL) & (C::CH - 1))) * 16);
                const uint32_t v_col16 = (uint32_t)(((lane_f % C::CH) ^ ((((r / C::RPL) & 3) << 2) & (C::CH - 1))) * 16);
                unsigned char* const kdst = lds + slot + (wave_u * C::NI + jn) * 1024;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(k_rsrc, (lds_void*)kdst, 16, row_off + k_col16, soff, 0, 0);
                __builtin_amdgcn_raw_ptr_buffer_load_lds(v_rsrc, (lds_void*)(kdst + C::V_RING), 16, row_off + v_col16, soff, 0, 0);
            }
        };
        // tile j: global memory -> ring slot j % NB, no registers in between
        auto fetch = [&](int j_) {
            const int j = __builtin_amdgcn_readfirstlane(j_);
            if (j < F) fetch_full(j, (uint32_t)(j & (NB - 1)) * C::T_BYTES); else fetch_masked(j);
            issued = j + 1;
        };
        // block until tile t has landed in LDS for the whole workgroup; tiles are
        // fetched in order, IPT load instructions per wavefront each
        int landed = -1;     // tiles up to this one are in LDS for every wavefront
        auto wait_landed = [&](int t) {
            landed = t;
            const int k = issued - 1 - t;
            if (k >= 3) wait_vm<3 * C::IPT>();
            else if (k == 2) wait_vm<2 * C::IPT>();
            else if (k == 1) wait_vm<C::IPT>();
            else wait_vm<0>();
            wg_barrier();
        };

        // masked tiles that fit the ring ahead of time
        while (issued < min(NB - 1, n_tiles)) fetch(issued);

        // ---- streaming-softmax state: one query row per lane --------------------
        f32x16 o[DB];
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int v = 0; v < 16; ++v) o[db][v] = 0.f;
        float m_ref = -INFINITY;   // reference value the exponentials are taken against (raw score units)
        float l_run = 0.f;         // this lane's share of the running sum

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

        bf16x8 p[4];      // probabilities of a tile as MFMA B operands, one per 16-key step

        // ---- full prefix tiles, software pipelined ---------------------------------
        // Issue order so far: Q, then K0 V0 K1 V1 K2 V2 K3.  The first step needs Q, K0, V0 and K1; with four
        // full tiles or more nothing else has been requested, and the last four half tiles may stay in flight.
        if (F >= NB) wait_vm<4 * C::NI>(); else wait_vm<0>();
        wg_barrier();
        landed = issued - 1;
        if (F > 0) {
            // prologue: scores of tile 0
            f32x16 sa[2], sb[2];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
                for (int v = 0; v < 16; ++v) sa[kb][v] = 0.f;
#pragma unroll
                for (int ks = 0; ks < KS; ++ks)
                    sa[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k_frag(0, kb, ks), qf[ks], sa[kb], 0, 0, 0);
            }

            // One pipelined step: probabilities and P V of tile i from s_cur while
            // the scores of tile i+1 go to s_nxt; K of tile i+4 and V of tile i+3 are requested.
            //   slots  0- 7  S(i+1) first 32 keys   ||  row maximum of tile i
            //   slots  8-15  S(i+1) second 32 keys  ||  exp of the first 32 keys
            //   slots 16-23  P V first 32 keys      ||  exp of the second 32 keys
            //   slots 24-31  P V second 32 keys
            // `par` is i % NB as a compile-time constant: ring slots become
            // immediate offsets of the LDS reads.  The scores of tile i+1 are
            // computed whether or not it is a full tile (from whatever its slot
            // holds); they are only used if it is.  On entry K up to tile i+1 and V up
            // to tile i have landed; on exit K up to tile i+2 and V up to tile i+1.
            auto step = [&](auto par, int i, f32x16 (&s_cur)[2], f32x16 (&s_nxt)[2]) {
                constexpr int P = decltype(par)::value;
                constexpr uint32_t KSLOT = (uint32_t)((P + 1) % NB) * C::T_BYTES;
                constexpr uint32_t VSLOT = (uint32_t)P * C::T_BYTES;
                // K of tile i+NB goes where K of tile i was (last read in the previous step, by the scores
                // computed ahead), V of tile i+NB-1 where V of tile i-1 was
                // (masked tiles are requested after the loop: their request code is long, and inside the
                // loop it costs registers the loop does not have: measured, 52..64 vector registers spilled)
                if (i + NB < F) fetch_k(i + NB, (uint32_t)P * C::T_BYTES);
                if (i + NB - 1 < F) {
                    fetch_v(i + NB - 1, (uint32_t)((P + NB - 1) % NB) * C::T_BYTES);
                    issued = i + NB;
                }
                auto kfrag = [&](int kb, int ks) {
                    return *reinterpret_cast<const bf16x8*>(lds + k_fragoff[ks] + (KSLOT + kb * 32 * D * 2));
                };
                // P V slot j of block kb: 16-key step j / DB, channel block j % DB
                auto vfrag = [&](int kb, int j) -> bf16x8 {
                    const int t4 = kb * 2 + j / DB, db = j % DB;
                    if (PACKED) return *reinterpret_cast<const bf16x8*>(lds + v_fragoff_ring + (VSLOT + t4 * (D * 32) + db * 512));
                    return v_frag_tr_at(vtr_off_ring + VSLOT, t4, db);
                };
                bf16x8 f[3];
                FDD_SCHED_FENCE();

                // ---- slots 0-7 ----
                float mx = -INFINITY;
                f[0] = kfrag(0, 0);
                f[1] = kfrag(0, 1);
#pragma unroll
                for (int v = 0; v < 16; ++v) s_nxt[0][v] = 0.f;
#pragma unroll
                for (int j = 0; j < KS; ++j) {
                    if (j + 2 < KS) f[(j + 2) % 3] = kfrag(0, j + 2);
                    s_nxt[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[j % 3], qf[j], s_nxt[0], 0, 0, 0);
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
                    typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
                    bf16x2 lo = {(__bf16)pr[0], (__bf16)pr[1]}, hi = {(__bf16)pr[2], (__bf16)pr[3]};
                    // the row sum is taken over the probabilities as they enter P V (rounded to bf16):
                    // numerator and denominator then see the same values, and a pair costs one instruction
                    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
                    acc = __builtin_amdgcn_fdot2_f32_bf16(lo, ones, acc, false);
                    acc = __builtin_amdgcn_fdot2_f32_bf16(hi, ones, acc, false);
                    uint32_t ulo = __builtin_bit_cast(uint32_t, lo), uhi = __builtin_bit_cast(uint32_t, hi);
                    FDD_PIN(ulo);
                    FDD_PIN(uhi);
                    FDD_PIN(acc);
                    pw[kb * 2 + e / 2][(e & 1) * 2] = ulo;
                    pw[kb * 2 + e / 2][(e & 1) * 2 + 1] = uhi;
                };
                FDD_SCHED_FENCE();

                // ---- slots 8-15 ----
                f[0] = kfrag(1, 0);
                f[1] = kfrag(1, 1);
#pragma unroll
                for (int v = 0; v < 16; ++v) s_nxt[1][v] = 0.f;
#pragma unroll
                for (int j = 0; j < KS; ++j) {
                    if (j + 2 < KS) f[(j + 2) % 3] = kfrag(1, j + 2);
                    s_nxt[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[j % 3], qf[j], s_nxt[1], 0, 0, 0);
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
                    FDD_SCHED_FENCE();
                }
                // K of tile i+2 and V of tile i+1 must have landed (both requested two steps ago); what this
                // step and the previous one requested may still be on its way
                if (i + 4 < F) wait_vm<4 * C::NI>();
                else if (i + 3 < F) wait_vm<3 * C::NI>();
                else if (i + 2 < F) wait_vm<C::NI>();
                else wait_vm<0>();
                wg_barrier();
            };
            const std::integral_constant<int, 0> r0;
            const std::integral_constant<int, 1> r1;
            const std::integral_constant<int, 2> r2;
            const std::integral_constant<int, 3> r3;
            for (int i = 0;;) {
                step(r0, i, sa, sb);
                if (++i == F) break;
                step(r1, i, sb, sa);
                if (++i == F) break;
                step(r2, i, sa, sb);
                if (++i == F) break;
                step(r3, i, sb, sa);
                if (++i == F) break;
            }
            landed = issued - 1;     // the last step waits for everything requested
        }

        // ---- masked tiles: ragged last prefix tile and the in-block tail ------------
        // On entry to iteration j tile j has landed.
        for (int j = F; j < n_tiles; ++j) {
            // the slots refilled here held tiles up to j-1, last read before the previous barrier
            while (issued < min(n_tiles, j + NB)) fetch(issued);
            if (landed < j) wait_landed(j);
            const Tile t = tile_at(j);
            const uint32_t kbase = (uint32_t)(j & (NB - 1)) * C::T_BYTES;
            const bool wave_active = wave_has_rows &&
                (t.rollout < 0 || (t.rollout >= wave_n_lo && t.rollout <= wave_n_hi));
            if (wave_active) {
                f32x16 s[2];
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) s[kb][v] = 0.f;
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks)
                        s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k_frag(kbase, kb, ks), qf[ks], s[kb], 0, 0, 0);
                }
                // register v of block kb is key kb*32 + (v/4)*8 + half*4 + v%4
                const bool row_sees = (t.rollout < 0) || (t.rollout == my_rollout);
                float mx = -INFINITY;
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int key = kb * 32 + (v >> 2) * 8 + half * 4 + (v & 3);
                        const bool later = a.causal && t.src == 2 && t.key0 + key > my_b;   // verify pass: causal inside the block
                        if (!row_sees || key >= t.valid || later) s[kb][v] = -INFINITY;
                        mx = fmaxf(mx, s[kb][v]);
                    }
                update_reference(fmaxf(mx, other_half(mx)));
                const float mc = ((m_ref == -INFINITY) ? 0.f : m_ref) * a.c;
                float acc = 0.f;
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const float pr = fast_exp2(fmaf(s[kb][v], a.c, -mc));
                        acc += pr;
                        p[kb * 2 + v / 8][v % 8] = (__bf16)pr;
                    }
                l_run += acc;
#pragma unroll
                for (int t4 = 0; t4 < 4; ++t4)
#pragma unroll
                    for (int db = 0; db < DB; ++db)
                        o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v_frag_tr_at(vtr_off_ring + kbase, t4, db), p[t4], o[db], 0, 0, 0);
            }
            if (j + 1 < n_tiles) wait_landed(j + 1); else wg_barrier();
        }
        const float m_run = m_ref;

        // ---- epilogue of the segment ------------------------------------------------
        const float l_tot = l_run + other_half(l_run);
        if (row_ok) {
            if (n_seg == 1) {
                const float inv = 1.f / l_tot;
                uint16_t* op = a.out + pb * a.o_bs + ((size_t)nb * a.Hq + (size_t)kh * a.G + g) * D;
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
                // Partial of this segment: the segment's own softmax average (o / l, rounded to bf16) and its
                // (m, l) in fp32.  The averages lie in the order of the accumulator registers,
                // [M-tile][segment][wavefront][register pair][lane] x 8 bf16, so every store instruction of a
                // wavefront writes 1 KB in one piece and the merge kernel reads them the same way.
                const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
                const size_t pseg = (size_t)M * a.max_seg + seg;
                u32x4* wo = reinterpret_cast<u32x4*>(a.ws_o) + (pseg * WAVES + wave) * (size_t)(2 * DB * 64) + lane;
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int v2 = 0; v2 < 2; ++v2) {
                        bf16x8 w;
#pragma unroll
                        for (int j = 0; j < 8; ++j) w[j] = (__bf16)(o[db][v2 * 8 + j] * inv);
                        wo[(db * 2 + v2) * 64] = __builtin_bit_cast(u32x4, w);
                    }
                if (half == 0) {
                    const size_t prow = pseg * MROWS + (wave * 32 + l32);
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
struct PackCfg {
    static constexpr int THREADS = 512;
    static constexpr int VROW = D * 2 + 64;              // padded row: conflict-free transposing reads
    static constexpr int V_BYTES = KT * VROW;
    static constexpr int K_PER_THREAD = KT * (D / 8) / THREADS;
    static constexpr int T_BYTES = KT * D * 2;
};

template <int D>
__global__ __launch_bounds__(512) void vt_pack_kernel(const uint16_t* __restrict__ pv_all, uint16_t* __restrict__ vt_all,
                                                       int Hkv, int TPF, long long p_bs, long long vt_bs)
{
    using C = PackCfg<D>;
    constexpr int DB = D / 32;
    __shared__ __align__(16) unsigned char tile[C::V_BYTES];
    // grid (tile, KV head of a problem of the batch)
    const int t = blockIdx.x, pb = blockIdx.y / Hkv, kh = blockIdx.y - pb * Hkv;
    const uint16_t* pv = pv_all + pb * p_bs;
    uint16_t* vt = vt_all + pb * vt_bs;
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

// ---------------------------------------------------------------------------
// Merge of the segments of an M-tile (log-sum-exp merge, paper-independent arithmetic of the split):
//   m* = max_s m_s,   W_s = l_s 2^((m_s - m*) c) / sum_t l_t 2^((m_t - m*) c),   out = sum_s W_s avg_s
// with avg_s the segment's own softmax average as the attention kernel left it (bf16, accumulator order).
// The sum over s runs in a fixed order, so results are reproducible.
// grid (M-tiles, 16 SG): a block of 256 threads = SG segment groups x 256/SG chunks of 8 channels of one
// wavefront's 32 rows; thread (sg, chunk) sums segments sg, sg + SG, .., four loads in flight, and the SG partial
// sums are added in the order sg = 0, 1, .. through LDS.  SG grows when rows are few and segments many (N = 1).
struct MergeArgs {
    const u32x4* ws_o;
    const float* ws_ml;
    uint16_t* out;
    const int32_t* qpos;
    long long o_bs;
    int Hq, Hkv, G, R, MT, NB;
    int max_seg, fixed_seg, TPU, base, rem;
    int SG;
    float c;
};

template <int D>
__global__ __launch_bounds__(256) void attn_merge_bf16_kernel(MergeArgs a)
{
    constexpr int DB = D / 32;
    constexpr int CPW = 2 * DB * 64;          // 16-byte chunks per wavefront of the attention kernel
    constexpr int CH = 8 * CPW;               // chunks per M-tile and segment
    extern __shared__ __align__(16) float smem[];
    const int tid = (int)threadIdx.x;
    const int M = (int)blockIdx.x;
    int n_seg = a.fixed_seg;
    if (n_seg == 0)     // same arithmetic as the attention kernel: workgroups whose unit range meets this M-tile
        n_seg = wg_of_unit((M + 1) * a.TPU - 1, a.base, a.rem) - wg_of_unit(M * a.TPU, a.base, a.rem) + 1;
    if (n_seg == 1) return;     // written in final form by its only segment
    const int khv = M / a.MT, mt = M - khv * a.MT;      // (problem of the batch, KV head), M-tile
    const int pb = khv / a.Hkv, kh = khv - pb * a.Hkv;
    const int CPB = 256 / a.SG;               // chunks per block: 32 .. 256, all of one wavefront (32 rows)
    const int c0 = (int)blockIdx.y * CPB;
    const int wave = c0 / CPW;
    const int row0 = mt * 256 + wave * 32;    // first stacked row of the block's 32 rows
    if (row0 >= a.R) return;

    // ---- this thread's chunk; the first four segments' averages are requested before anything else, so that
    // their latency and that of the (m, l) pairs below overlap ------------------------------------
    const int sg = tid / CPB, cl = tid - sg * CPB;
    const int cidx = c0 + cl;                          // chunk inside the M-tile: [wave][register pair][lane]
    const int lane = cidx & 63, i2 = (cidx >> 6) % (2 * DB);
    const int r = lane & 31, half = lane >> 5;
    const bool live = row0 + r < a.R;
    const u32x4* src = a.ws_o + ((size_t)M * a.max_seg) * CH + cidx;
    u32x4 x[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int s = sg + u * a.SG;
        x[u] = u32x4{0u, 0u, 0u, 0u};
        if (live && s < n_seg) x[u] = src[(size_t)s * CH];
    }

    // ---- weights of the segments, per row: 8 threads per row ----------------------------------
    float* const W = smem;                            // [32][n_seg]
    {
        const int rr = tid >> 3, j = tid & 7;
        const bool live_r = row0 + rr < a.R;
        const float* ml = a.ws_ml + (((size_t)M * a.max_seg) * 256 + wave * 32 + rr) * 2;
        float mx = -INFINITY;
        for (int s = j; s < n_seg; s += 8) {
            float2 y = make_float2(-INFINITY, 0.f);
            if (live_r) y = *reinterpret_cast<const float2*>(ml + (size_t)s * 512);
            if (!(y.y > 0.f)) y.x = -INFINITY;        // a segment that saw no key of this row
            W[rr * n_seg + s] = y.x;
            smem[32 * n_seg + rr * n_seg + s] = y.y;
            mx = fmaxf(mx, y.x);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 1, 64));
        mx = fmaxf(mx, __shfl_xor(mx, 2, 64));
        mx = fmaxf(mx, __shfl_xor(mx, 4, 64));
        const float mref = mx == -INFINITY ? 0.f : mx;
        float sum = 0.f;
        for (int s = j; s < n_seg; s += 8) {
            const float w = smem[32 * n_seg + rr * n_seg + s] * exp2f((W[rr * n_seg + s] - mref) * a.c);
            W[rr * n_seg + s] = w;
            sum += w;
        }
        sum += __shfl_xor(sum, 1, 64);
        sum += __shfl_xor(sum, 2, 64);
        sum += __shfl_xor(sum, 4, 64);
        const float inv = sum > 0.f ? 1.f / sum : 0.f;
        for (int s = j; s < n_seg; s += 8) W[rr * n_seg + s] *= inv;
    }
    __syncthreads();

    // ---- weighted sum of the segments' averages -------------------------------------------------
    float acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = 0.f;
    if (live) {
        for (int s0 = sg; s0 < n_seg; s0 += 4 * a.SG) {
            // the next four segments of this thread are requested before the current four are summed
            u32x4 nx[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int s = s0 + (4 + u) * a.SG;
                nx[u] = u32x4{0u, 0u, 0u, 0u};
                if (s < n_seg) nx[u] = src[(size_t)s * CH];
            }
            float w[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int s = s0 + u * a.SG;
                w[u] = s < n_seg ? W[r * n_seg + s] : 0.f;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    // (a weight of 0 belongs to a segment without a key of this row: its average is 0 as well)
                    acc[2 * j] = fmaf(__uint_as_float(x[u][j] << 16), w[u], acc[2 * j]);
                    acc[2 * j + 1] = fmaf(__uint_as_float(x[u][j] & 0xffff0000u), w[u], acc[2 * j + 1]);
                }
#pragma unroll
            for (int u = 0; u < 4; ++u) x[u] = nx[u];
        }
    }
    if (a.SG > 1) {
        float* const red = smem + 2 * 32 * n_seg;     // [SG][CPB][8]
        __syncthreads();
#pragma unroll
        for (int j = 0; j < 8; ++j) red[(sg * CPB + cl) * 8 + j] = acc[j];
        __syncthreads();
        if (sg != 0) return;
        for (int k = 1; k < a.SG; ++k)
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[j] += red[(k * CPB + cl) * 8 + j];
    }
    if (!live) return;
    const int row = row0 + r;
    const int sel = row / a.G, g = row - sel * a.G;
    const int nb = a.qpos ? min(max(a.qpos[sel], 0), a.NB - 1) : sel;
    const int db = i2 >> 1, v2 = i2 & 1;
    uint16_t* op = a.out + pb * a.o_bs + ((size_t)nb * a.Hq + (size_t)kh * a.G + g) * D + db * 32 + v2 * 16 + half * 4;
    typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
    bf16x4 lo, hi;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        lo[j] = (__bf16)acc[j];
        hi[j] = (__bf16)acc[4 + j];
    }
    *reinterpret_cast<bf16x4*>(op) = lo;
    *reinterpret_cast<bf16x4*>(op + 8) = hi;
}

template <int D, int WAVES, bool PACKED>
hipError_t launch(const Args& a, bool pack_now, hipStream_t stream, hipEvent_t before_main)
{
    using C = Cfg<D, WAVES>;
    const size_t lds_bytes = C::LDS_BYTES;
    const auto kern = &attn_bf16_kernel<D, WAVES, PACKED>;
    // the LDS limit of this instantiation is raised once per device (bit d of `done`: device d)
    static std::atomic<uint64_t> done{0};
    int dev = 0;
    if (hipError_t e = hipGetDevice(&dev); e != hipSuccess) return e;
    const uint64_t bit = 1ull << (dev & 63);
    if (!(done.load(std::memory_order_acquire) & bit)) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
        done.fetch_or(bit, std::memory_order_release);
    }
    if (PACKED && pack_now) {
        hipLaunchKernelGGL(vt_pack_kernel<D>, dim3(a.TPF, a.Hkv * a.batch), dim3(512), 0, stream, a.pv,
                           const_cast<uint16_t*>(a.vt), a.Hkv, a.TPF, a.p_bs, a.vt_bs);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (before_main) {
        hipError_t e = hipEventRecord(before_main, stream);
        if (e != hipSuccess) return e;
    }
    const int grid = a.per_xcd * kNumXCD;   // padded so that every XCD gets the same count
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
    a.ws_o = ws;
    a.ws_ml = reinterpret_cast<float*>(ws + plan.ws_o_bytes);
    const bool pack_now = plan.packed && !p.prefix_v_packed;
    a.vt = pack_now ? reinterpret_cast<const uint16_t*>(ws + plan.ws_o_bytes + plan.ws_ml_bytes)
                    : static_cast<const uint16_t*>(p.prefix_v_packed);
    a.ek = static_cast<const uint16_t*>(p.ext_k);
    a.ev = static_cast<const uint16_t*>(p.ext_v);
    a.E = p.E; a.Ecap = p.ext_capacity;
    a.batch = p.batch > 1 ? p.batch : 1;
    a.q_bs = p.q_batch_stride; a.p_bs = p.prefix_batch_stride; a.b_bs = p.block_batch_stride;
    a.e_bs = p.ext_batch_stride; a.o_bs = p.out_batch_stride;
    // packed V: the caller's stride, or the in-call copies lying back to back in the workspace
    a.vt_bs = pack_now ? (long long)p.Hkv * (p.L / 64) * 64 * p.D : (long long)(p.packed_batch_stride / 2);
    a.N = p.N; a.B = p.B; a.L = p.L; a.Hq = p.Hq; a.Hkv = p.Hkv;
    a.G = plan.G; a.R = plan.R; a.MT = plan.MT; a.TP = plan.TP; a.TPF = p.L / 64;
    a.TPU = plan.TPU; a.W = plan.W; a.max_seg = plan.max_seg; a.S = plan.uniform;
    a.per_xcd = (plan.W + kNumXCD - 1) / kNumXCD;
    a.base = (int)(plan.U / plan.W); a.rem = (int)(plan.U % plan.W);
    a.causal = (p.flags & FDD_ATTN_CAUSAL_BLOCK) ? 1 : 0;
    a.c = scale * 1.4426950408889634f;
    a.ttpr = (p.E + 63) / 64 + (p.B + 63) / 64;
    a.qpos = p.n_q_positions > 0 ? p.q_positions : nullptr;
    a.NB = p.N * p.B;
    a.dMT = make_fastdiv((uint32_t)a.MT);
    a.dS = make_fastdiv((uint32_t)(a.S > 0 ? a.S : 1));
    a.dTPU = make_fastdiv((uint32_t)a.TPU);
    a.dHkv = make_fastdiv((uint32_t)a.Hkv);
    a.dG = make_fastdiv((uint32_t)a.G);
    a.dB = make_fastdiv((uint32_t)a.B);
    a.dBG = make_fastdiv((uint32_t)(a.B * a.G));
    a.dTTPR = make_fastdiv((uint32_t)a.ttpr);
    a.dBase = make_fastdiv((uint32_t)(a.base > 0 ? a.base : 1));
    a.dBase1 = make_fastdiv((uint32_t)(a.base + 1));
    a.dPerXcd = make_fastdiv((uint32_t)a.per_xcd);
    // (with 2..16 pieces of 32 units or more a shift of 3 % is at least one unit)
    a.w_even = 100;
    a.w_odd = (a.S >= 2 && a.S <= 16 && a.TPU >= 32 * a.S) ? ODD_XCD_WEIGHT : 100;
    if (plan.mtile_rows != 256) return hipErrorInvalidValue;
    if (plan.packed)
        return p.D == 128 ? launch<128, 8, true>(a, pack_now, s, before_main) : launch<64, 8, true>(a, pack_now, s, before_main);
    return p.D == 128 ? launch<128, 8, false>(a, false, s, before_main) : launch<64, 8, false>(a, false, s, before_main);
}

hipError_t launch_attn_merge_bf16(const fdd_attn_params& p, const AttnPlan& plan, float scale, hipStream_t s)
{
    MergeArgs a;
    a.ws_o = static_cast<const u32x4*>(p.workspace);
    a.ws_ml = reinterpret_cast<const float*>(static_cast<const char*>(p.workspace) + plan.ws_o_bytes);
    a.out = static_cast<uint16_t*>(p.out);
    a.qpos = p.n_q_positions > 0 ? p.q_positions : nullptr;
    a.o_bs = p.out_batch_stride;
    const int batch = p.batch > 1 ? p.batch : 1;
    a.Hq = p.Hq; a.Hkv = p.Hkv; a.G = plan.G; a.R = plan.R; a.MT = plan.MT; a.NB = p.N * p.B;
    a.max_seg = plan.max_seg; a.fixed_seg = plan.uniform; a.TPU = plan.TPU;
    a.base = (int)(plan.U / plan.W); a.rem = (int)(plan.U % plan.W);
    a.c = scale * 1.4426950408889634f;
    // more threads per chunk when the rows are few and the segments many
    const long long rows = (long long)p.Hkv * batch * plan.R;
    const int seg_hint = plan.uniform > 0 ? plan.uniform : plan.max_seg;
    int sg = 1;
    while (sg < 8 && sg * 2 <= seg_hint && rows * sg < 16384) sg *= 2;
    a.SG = sg;
    const int chunks = 8 * 2 * (p.D / 32) * 64;
    const size_t smem = ((size_t)2 * 32 * plan.max_seg + (sg > 1 ? (size_t)256 * 8 : 0)) * sizeof(float);
    if (smem > 60 * 1024 || plan.mtile_rows != 256) return hipErrorInvalidValue;
    const dim3 grid((unsigned)(p.Hkv * batch * plan.MT), (unsigned)(chunks / (256 / sg)));
    if (p.D == 128) hipLaunchKernelGGL(attn_merge_bf16_kernel<128>, grid, dim3(256), smem, s, a);
    else hipLaunchKernelGGL(attn_merge_bf16_kernel<64>, grid, dim3(256), smem, s, a);
    return hipGetLastError();
}

hipError_t launch_prefix_pack(const void* prefix_v, int L, int Hkv, int D, void* packed, hipStream_t s)
{
    const int TPF = L / KT;
    if (TPF == 0) return hipSuccess;
    const uint16_t* src = static_cast<const uint16_t*>(prefix_v);
    uint16_t* dst = static_cast<uint16_t*>(packed);
    if (D == 128) hipLaunchKernelGGL(vt_pack_kernel<128>, dim3(TPF, Hkv), dim3(512), 0, s, src, dst, Hkv, TPF, 0ll, 0ll);
    else hipLaunchKernelGGL(vt_pack_kernel<64>, dim3(TPF, Hkv), dim3(512), 0, s, src, dst, Hkv, TPF, 0ll, 0ll);
    return hipGetLastError();
}

}  // namespace fdd
