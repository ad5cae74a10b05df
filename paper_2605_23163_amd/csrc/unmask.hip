// Confidence-threshold unmasking of one block per rollout.
//
// One iteration of "iteratively unmasks value positions" (paper, "Section
// Diffusion (SD)"): masked, non-scaffold positions are the only ones touched
// (Eq. 2; visible tokens stay fixed).  For each such position the row of V
// logits is reduced to (arg max, largest softmax probability); a position
// commits when that probability reaches tau, and a block that would commit
// nothing commits its most confident eligible position.
//
// Two kernels:
//   vocab_reduce  streams the logits rows of eligible positions once.  A row
//                 is cut into `vsplits` pieces so that a few hundred rows
//                 still fill 256 CUs; each piece is reduced by one workgroup
//                 to (max, lowest arg max, sum exp(x - max)) with a one-pass
//                 running-maximum sum.  (value, index) pairs are ordered by
//                 value descending then index ascending through every
//                 in-thread, cross-lane and cross-wave stage, so ties of
//                 stored values (frequent in bf16) always resolve to the
//                 lowest id.  Workgroups of non-eligible rows exit at once
//                 and read nothing.
//   vocab_sample  the sampled verifier's sibling of vocab_reduce: the value
//                 reduced is the Gumbel-max key of every vocabulary entry
//                 (a Philox-4x32-10 word per entry, two polynomial log2, one
//                 fused multiply-add), so the pass is bound by the vector ALUs
//                 rather than by HBM.
//   block_select  one workgroup per rollout: merges the pieces of each
//                 position in a fixed order (sum finished in fp64), applies
//                 the tau test and the forced single commit, and writes
//                 tokens / mask / confidences.
#include "fdd_internal.h"

namespace fdd {
namespace {

constexpr float LOG2E = 1.4426950408889634f;
constexpr int RTHREADS = 256;
constexpr int UNROLL = 6;            // 16-byte loads in flight per thread
constexpr int PIECE_KB = 64;         // a row is cut into pieces of at least this size ...
constexpr int PIECE_KB_ARGMAX = 32;  // ... and of this size in the pass that takes no sums (measured: 8 pieces of a
                                     // 297 KB row are 1.5 us per call faster there than 4, and 1..2 us slower with the sums)
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct Partial {
    float m;
    int32_t arg;
    float s;
    int32_t pad;
};

struct Args {
    const void* logits;
    const uint8_t* scaffold;
    uint8_t* mask;
    int32_t* tokens;
    float* conf;
    int32_t* n_unmasked;
    uint8_t* committed;
    Partial* ws;
    const int32_t* draft;   // verify pass only
    // K/V refresh of the committed positions (unmask step only): row (token mod T) of the tables, or no refresh
    const u32x4* rf_tk;
    const u32x4* rf_tv;
    u32x4* rf_bk;
    u32x4* rf_bv;
    int rf_T, rf_row_vecs;  // table rows; 16-byte pieces per K/V row (0: no refresh)
    int N, B, vsplits;
    long long V;
    float tau;
    float c;                // sampled verifier: log2(e) / temperature
    uint32_t seed_lo, seed_hi;
};

struct Run {
    float m;      // running maximum
    int idx;      // lowest index attaining it
    float s;      // sum of 2^((x - m) log2 e) over what was seen
};

// A thread's running sum takes its terms as 2^(x c - fl(m c)), c = log2 e, with one fused
// multiply-add each.  fl(m c) is off from m c by up to half an ulp, which scales every term
// by the same 2^(m c - fl(m c)): harmless as long as the whole sum is relative to the same
// fl(m c).  So a new maximum rescales the sum by 2^(fl(m_old c) - fl(m_new c)), the
// difference of the rounded products, and the common factor is taken out once, by
// `settle`, before sums of different threads meet.
struct ThreadRun {
    Run r;
    float mc;     // fl(r.m * log2 e)
};

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// `b` is merged into `a`; on equal maxima the lower index wins.
__device__ __forceinline__ void merge(Run& a, const Run& b)
{
    const bool take_b = (b.m > a.m) || (b.m == a.m && b.idx < a.idx);
    const float M = fmaxf(a.m, b.m);
    const float sa = (a.m == M) ? a.s : a.s * fast_exp2((a.m - M) * LOG2E);
    const float sb = (b.m == M) ? b.s : b.s * fast_exp2((b.m - M) * LOG2E);
    a.s = sa + sb;
    a.m = M;
    if (take_b) a.idx = b.idx;
}

// SUM = false: only (max, arg max) are kept (the greedy verifier needs no probabilities)
template <int VEC, bool SUM>
__device__ __forceinline__ void absorb(ThreadRun& t, const float (&x)[VEC], int v0)
{
    Run& r = t.r;
    float cm = x[0];
#pragma unroll
    for (int j = 1; j < VEC; ++j) cm = fmaxf(cm, x[j]);
    if (cm > r.m) {
        // this thread walks the row in ascending order, so a strictly larger
        // value is the only way its arg max can move
        if (SUM) {
            const float mc_new = cm * LOG2E;
            r.s *= fast_exp2(t.mc - mc_new);      // (-inf - finite at the start: the sum is still 0)
            t.mc = mc_new;
        }
        r.m = cm;
        int first = VEC - 1;
#pragma unroll
        for (int j = VEC - 2; j >= 0; --j) first = (x[j] == cm) ? j : first;
        r.idx = v0 + first;
    }
    if (!SUM) return;
    // (a thread that has only met -inf so far takes its terms against 0: 2^(-inf) = 0, never inf - inf)
    const float mc = (t.mc == -INFINITY) ? 0.f : t.mc;
    float acc = 0.f;
#pragma unroll
    for (int j = 0; j < VEC; ++j) acc += fast_exp2(fmaf(x[j], LOG2E, -mc));
    r.s += acc;
}

// the sum as taken against m itself (see ThreadRun)
__device__ __forceinline__ Run settle(const ThreadRun& t)
{
    Run r = t.r;
    if (r.m != -INFINITY) r.s *= fast_exp2(-fmaf(r.m, LOG2E, -t.mc));
    return r;
}

__device__ __forceinline__ float bf16_to_f32(uint32_t bits16) { return __uint_as_float(bits16 << 16); }

// Workgroups are dealt to the 8 XCDs round-robin by launch index, and a workgroup whose row is
// not eligible leaves at once.  With (row, piece) = (index / vsplits, index % vsplits) an XCD
// would always get rows of the same residue, and a scaffold pattern that repeats from rollout
// to rollout (it does: the schema is shared) would load the XCDs unequally.  So each group of 8
// consecutive indices is rotated, by an amount that changes from group to group, from 8 groups to the
// next 8 and from 64 to the next 64 (a rotation by the group's number alone repeats with the pattern:
// config 5's 720 eligible rows of 4 pieces then give the XCDs 304..416 workgroups instead of 360 each).
__device__ __forceinline__ unsigned unit_of_workgroup()
{
    const unsigned u = blockIdx.x, g = u >> 3;
    if ((g << 3) + 8u > gridDim.x) return u;           // a last, incomplete group stays as it is
    return (g << 3) + ((u + g + (g >> 3) + (g >> 6) + (g >> 9)) & 7u);
}

// T = uint16_t (bf16 bits) or float; SUM = false leaves (max, arg max) only and a sum of 0
template <typename T, bool SUM>
__global__ __launch_bounds__(RTHREADS) void vocab_reduce_kernel(Args a)
{
    constexpr int VEC = 16 / sizeof(T);
    const unsigned unit = unit_of_workgroup();
    const int row = unit / a.vsplits;
    if (a.mask[row] != 1 || (a.scaffold && a.scaffold[row])) return;
    const int piece = unit % a.vsplits;
    const long long per = (a.V + a.vsplits - 1) / a.vsplits;
    const long long v_lo = piece * per;
    const long long v_hi = min(a.V, v_lo + per);
    const T* base = static_cast<const T*>(a.logits) + (size_t)row * (size_t)a.V;
    const int tid = threadIdx.x;

    ThreadRun tr;
    tr.r.m = -INFINITY;
    tr.r.idx = 0x7fffffff;
    tr.r.s = 0.f;
    tr.mc = -INFINITY;

    if (v_lo < v_hi) {
        // leading elements up to the first 16-byte boundary, then whole
        // vectors, then the remainder; each thread visits ascending indices
        const size_t e_lo = (size_t)row * (size_t)a.V + (size_t)v_lo;
        long long head = (long long)((VEC - (e_lo % VEC)) % VEC);
        if (head > v_hi - v_lo) head = v_hi - v_lo;
        const long long body0 = v_lo + head;
        const long long nvec = (v_hi - body0) / VEC;
        const long long tail0 = body0 + nvec * VEC;

        if (tid < head) {
            float x[1] = {sizeof(T) == 2 ? bf16_to_f32(((const uint16_t*)base)[v_lo + tid]) : ((const float*)base)[v_lo + tid]};
            absorb<1, SUM>(tr, x, (int)(v_lo + tid));
        }
        const u32x4* vp = reinterpret_cast<const u32x4*>(base + body0);
        auto widen = [&](const u32x4& raw, float (&x)[VEC]) {
            if (sizeof(T) == 2) {
                const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    x[2 * j] = __uint_as_float(w[j] << 16);
                    x[2 * j + 1] = __uint_as_float(w[j] & 0xffff0000u);
                }
            } else {
                x[0] = __uint_as_float(raw.x);
                x[1] = __uint_as_float(raw.y);
                x[2] = __uint_as_float(raw.z);
                x[3] = __uint_as_float(raw.w);
            }
        };
        // UNROLL independent 16-byte loads in flight per thread, absorbed in ascending order
        long long i = tid;
        for (; i + (UNROLL - 1) * RTHREADS < nvec; i += UNROLL * RTHREADS) {
            u32x4 raw[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) raw[u] = __builtin_nontemporal_load(vp + i + u * RTHREADS);
            // all of them are requested before the first is waited for (left to itself the scheduler waits
            // for the first after two requests and only then issues the rest: two latencies per group)
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                float x[VEC];
                widen(raw[u], x);
                absorb<VEC, SUM>(tr, x, (int)(body0 + (i + u * RTHREADS) * VEC));
            }
        }
        if (i < nvec) {
            // the ragged last group: its loads are requested together as well
            u32x4 raw[UNROLL - 1];
#pragma unroll
            for (int u = 0; u < UNROLL - 1; ++u)
                if (i + u * RTHREADS < nvec) raw[u] = __builtin_nontemporal_load(vp + i + u * RTHREADS);
#pragma unroll
            for (int u = 0; u < UNROLL - 1; ++u) {
                if (i + u * RTHREADS < nvec) {
                    float x[VEC];
                    widen(raw[u], x);
                    absorb<VEC, SUM>(tr, x, (int)(body0 + (i + u * RTHREADS) * VEC));
                }
            }
        }
        const long long ntail = v_hi - tail0;
        if (tid < ntail) {
            float x[1] = {sizeof(T) == 2 ? bf16_to_f32(((const uint16_t*)base)[tail0 + tid]) : ((const float*)base)[tail0 + tid]};
            // tail indices are larger than anything this thread saw before
            absorb<1, SUM>(tr, x, (int)(tail0 + tid));
        }
    }

    // wavefront reduction, then across the 4 wavefronts through LDS
    Run r = SUM ? settle(tr) : tr.r;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        Run o;
        o.m = __shfl_xor(r.m, off, 64);
        o.idx = __shfl_xor(r.idx, off, 64);
        o.s = __shfl_xor(r.s, off, 64);
        merge(r, o);
    }
    __shared__ Run part[RTHREADS / 64];
    if ((tid & 63) == 0) part[tid >> 6] = r;
    __syncthreads();
    if (tid == 0) {
        Run t = part[0];
#pragma unroll
        for (int w = 1; w < RTHREADS / 64; ++w) merge(t, part[w]);
        Partial p;
        p.m = t.m;
        p.arg = t.idx;
        p.s = t.s;
        p.pad = 0;
        a.ws[(size_t)row * a.vsplits + piece] = p;
    }
}

// ---- sampled verifier ------------------------------------------------------
// The arithmetic below is the definition of the sampler (see fdd_verify_step
// in the public header): every operation is written out as one exactly
// rounded binary32 operation and must not be contracted or reassociated.

// Philox-4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw: "Parallel random
// numbers: as easy as 1, 2, 3", SC'11): counter (c0, c1, 0, 0), key (k0, k1).
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t k0, uint32_t k1, uint32_t (&out)[4])
{
    uint32_t c2 = 0u, c3 = 0u;
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        c0 = hi1 ^ c1 ^ k0;
        c1 = lo1;
        c2 = hi0 ^ c3 ^ k1;
        c3 = lo0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// log2 of a positive normal float: x = m 2^e, m in [1/sqrt 2, sqrt 2), e + f P(f) with f = m - 1
__device__ __forceinline__ float flog2_def(float x)
{
    const uint32_t bits = __float_as_uint(x);
    int e = (int)((bits >> 23) & 255u) - 127;
    float m = __uint_as_float((bits & 0x7fffffu) | 0x3f800000u);
    if (m > 1.41421354f) { m = __fmul_rn(m, 0.5f); e += 1; }
    const float f = __fsub_rn(m, 1.0f);
    float p = 0.12614846229553223f;
    p = __fmaf_rn(p, f, -0.20742103457450867f);
    p = __fmaf_rn(p, f, 0.21566985547542572f);
    p = __fmaf_rn(p, f, -0.23892034590244293f);
    p = __fmaf_rn(p, f, 0.2879183292388916f);
    p = __fmaf_rn(p, f, -0.36070483922958374f);
    p = __fmaf_rn(p, f, 0.48091059923171997f);
    p = __fmaf_rn(p, f, -0.7213473320007324f);
    p = __fmaf_rn(p, f, 1.4426950216293335f);
    return __fmaf_rn(f, p, (float)e);
}

__device__ __forceinline__ float gumbel_key(float x, float c, uint32_t r)
{
    const float u = __fmul_rn(__fadd_rn((float)(r >> 9), 0.5f), 1.1920928955078125e-07f);
    const float a = -flog2_def(u);
    const float g = -flog2_def(a);
    return __fmaf_rn(x, c, g);
}

struct Best {
    float k;
    int idx;
};
__device__ __forceinline__ void take(Best& a, float k, int idx)
{
    if (k > a.k || (k == a.k && idx < a.idx)) { a.k = k; a.idx = idx; }
}

// Same work split as vocab_reduce; leaves (largest key, lowest id attaining it) per piece.
template <typename T>
__global__ __launch_bounds__(RTHREADS) void vocab_sample_kernel(Args a)
{
    constexpr int VEC = 16 / sizeof(T);
    const unsigned unit = unit_of_workgroup();
    const int row = unit / a.vsplits;
    if (a.mask[row] != 1 || (a.scaffold && a.scaffold[row])) return;
    const int piece = unit % a.vsplits;
    const long long per = (a.V + a.vsplits - 1) / a.vsplits;
    const long long v_lo = piece * per;
    const long long v_hi = min(a.V, v_lo + per);
    const T* base = static_cast<const T*>(a.logits) + (size_t)row * (size_t)a.V;
    const int tid = threadIdx.x;
    Best r;
    r.k = -INFINITY;
    r.idx = 0x7fffffff;

    auto one = [&](long long v) {     // a single entry: its own generator block
        const float x = sizeof(T) == 2 ? bf16_to_f32(((const uint16_t*)base)[v]) : ((const float*)base)[v];
        uint32_t w[4];
        philox4x32_10((uint32_t)(v >> 2), (uint32_t)row, a.seed_lo, a.seed_hi, w);
        take(r, gumbel_key(x, a.c, w[v & 3]), (int)v);
    };
    if (v_lo < v_hi) {
        const size_t e_lo = (size_t)row * (size_t)a.V + (size_t)v_lo;
        long long head = (long long)((VEC - (e_lo % VEC)) % VEC);
        if (head > v_hi - v_lo) head = v_hi - v_lo;
        const long long body0 = v_lo + head;
        const long long nvec = (v_hi - body0) / VEC;
        const long long tail0 = body0 + nvec * VEC;
        if (tid < head) one(v_lo + tid);
        const u32x4* vp = reinterpret_cast<const u32x4*>(base + body0);
        const bool quads = (body0 & 3) == 0;      // a 16-byte vector then holds whole generator blocks
        for (long long i = tid; i < nvec; i += RTHREADS) {
            const u32x4 raw = __builtin_nontemporal_load(vp + i);
            const long long v0 = body0 + i * VEC;
            float x[VEC];
            if (sizeof(T) == 2) {
                const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    x[2 * j] = __uint_as_float(w[j] << 16);
                    x[(2 * j + 1) % VEC] = __uint_as_float(w[j] & 0xffff0000u);
                }
            } else {
                x[0] = __uint_as_float(raw.x);
                x[1] = __uint_as_float(raw.y);
                x[2 % VEC] = __uint_as_float(raw.z);
                x[3 % VEC] = __uint_as_float(raw.w);
            }
            if (quads) {
#pragma unroll
                for (int q = 0; q < VEC / 4; ++q) {
                    uint32_t w[4];
                    philox4x32_10((uint32_t)((v0 >> 2) + q), (uint32_t)row, a.seed_lo, a.seed_hi, w);
#pragma unroll
                    for (int j = 0; j < 4; ++j) take(r, gumbel_key(x[q * 4 + j], a.c, w[j]), (int)(v0 + q * 4 + j));
                }
            } else {
#pragma unroll
                for (int j = 0; j < VEC; ++j) {
                    uint32_t w[4];
                    philox4x32_10((uint32_t)((v0 + j) >> 2), (uint32_t)row, a.seed_lo, a.seed_hi, w);
                    take(r, gumbel_key(x[j], a.c, w[(v0 + j) & 3]), (int)(v0 + j));
                }
            }
        }
        const long long ntail = v_hi - tail0;
        if (tid < ntail) one(tail0 + tid);
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const float ok = __shfl_xor(r.k, off, 64);
        const int oi = __shfl_xor(r.idx, off, 64);
        take(r, ok, oi);
    }
    __shared__ Best part[RTHREADS / 64];
    if ((tid & 63) == 0) part[tid >> 6] = r;
    __syncthreads();
    if (tid == 0) {
        Best t = part[0];
#pragma unroll
        for (int w = 1; w < RTHREADS / 64; ++w) take(t, part[w].k, part[w].idx);
        Partial p;
        p.m = t.k;
        p.arg = t.idx;
        p.s = 0.f;
        p.pad = 0;
        a.ws[(size_t)row * a.vsplits + piece] = p;
    }
}

constexpr int STHREADS = 64;   // one wavefront per rollout: no LDS, no workgroup barrier

__global__ __launch_bounds__(STHREADS) void block_select_kernel(Args a)
{
    const int n = blockIdx.x;
    const int tid = threadIdx.x;
    const double tau = (double)a.tau;

    int count = 0;
    double best_conf = -1.0;     // confidences are positive
    int best_b = 0x7fffffff;
    int best_tok = -1;

    // the wavefront refreshes the K/V row of position i, which now holds token `tok` (see fdd_block_kv_update)
    auto refresh_row = [&](size_t i, int tok) {
        int t = tok % a.rf_T;
        if (t < 0) t += a.rf_T;
        for (int c = tid; c < a.rf_row_vecs; c += STHREADS) {
            a.rf_bk[i * a.rf_row_vecs + c] = a.rf_tk[(size_t)t * a.rf_row_vecs + c];
            a.rf_bv[i * a.rf_row_vecs + c] = a.rf_tv[(size_t)t * a.rf_row_vecs + c];
        }
    };

    for (int b0 = 0; b0 < a.B; b0 += STHREADS) {     // lane `tid` takes position b0 + tid (ascending per lane)
        const int b = b0 + tid;
        const size_t i = (size_t)n * a.B + (b < a.B ? b : 0);
        // The first pieces' records are requested together with the mask bytes, not after them: whether the
        // position is eligible is known one memory round trip later, and the records are then already there.
        // (records of positions that are not eligible hold whatever an earlier call left; they are not used)
        constexpr int PRE = 4;
        const u32x4* pr = reinterpret_cast<const u32x4*>(a.ws + i * a.vsplits);
        u32x4 rec[PRE];
#pragma unroll
        for (int s = 0; s < PRE; ++s) rec[s] = s < a.vsplits ? pr[s] : u32x4{0u, 0u, 0u, 0u};
        const bool eligible = b < a.B && a.mask[i] == 1 && !(a.scaffold && a.scaffold[i]);
        float conf_out = -INFINITY;
        uint8_t com = 0;
        int arg = -1;
        if (eligible) {
            auto unpack = [](const u32x4& r) {
                Partial q;
                q.m = __uint_as_float(r.x); q.arg = (int)r.y; q.s = __uint_as_float(r.z); q.pad = 0;
                return q;
            };
            const Partial* p = a.ws + i * a.vsplits;
            // pieces cover ascending index ranges: strict '>' keeps the lowest id
            float M = unpack(rec[0]).m;
            arg = unpack(rec[0]).arg;
#pragma unroll
            for (int s = 1; s < PRE; ++s) {
                const Partial q = unpack(rec[s]);
                if (s < a.vsplits && q.m > M) { M = q.m; arg = q.arg; }
            }
            for (int s = PRE; s < a.vsplits; ++s)
                if (p[s].m > M) { M = p[s].m; arg = p[s].arg; }
            // sum of the pieces' fp32 sums, rescaled to the row maximum, finished in fp64
            double z = 0.0;
#pragma unroll
            for (int s = 0; s < PRE; ++s) {
                const Partial q = unpack(rec[s]);
                if (s < a.vsplits && q.s > 0.f) z += (double)(q.s * fast_exp2((q.m - M) * LOG2E));
            }
            for (int s = PRE; s < a.vsplits; ++s)
                if (p[s].s > 0.f) z += (double)(p[s].s * fast_exp2((p[s].m - M) * LOG2E));
            const double conf = 1.0 / z;
            conf_out = (float)conf;
            if (conf >= tau) {
                a.tokens[i] = arg;
                a.mask[i] = 0;
                com = 1;
                ++count;
            }
            if (conf > best_conf) { best_conf = conf; best_b = b; best_tok = arg; }   // ascending b per thread
        }
        if (b < a.B) {
            a.conf[i] = conf_out;
            if (a.committed) a.committed[i] = com;
        }
        if (a.rf_row_vecs > 0) {
            unsigned long long m = __ballot(com != 0);
            while (m) {
                const int j = __ffsll((long long)m) - 1;
                m &= m - 1;
                refresh_row((size_t)n * a.B + b0 + j, __shfl(arg, j, 64));
            }
        }
    }
    // wavefront reduction: commits are summed; the best candidate is the one of
    // highest confidence, lowest position on ties
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        count += __shfl_xor(count, off, 64);
        const double oc = __shfl_xor(best_conf, off, 64);
        const int ob = __shfl_xor(best_b, off, 64);
        const int ot = __shfl_xor(best_tok, off, 64);
        if (oc > best_conf || (oc == best_conf && ob < best_b)) { best_conf = oc; best_b = ob; best_tok = ot; }
    }
    // (count and the best candidate are now the same in every lane)
    if (count == 0 && best_tok >= 0) {
        // nothing reached tau: commit the most confident eligible position
        const size_t i = (size_t)n * a.B + best_b;
        if (tid == 0) {
            a.tokens[i] = best_tok;
            a.mask[i] = 0;
            if (a.committed) a.committed[i] = 1;
        }
        if (a.rf_row_vecs > 0) refresh_row(i, best_tok);
        count = 1;
    }
    if (tid == 0 && a.n_unmasked) a.n_unmasked[n] = count;
}

// Accept scan of scaffold speculative decoding: one wavefront per rollout.
// Draft positions are visited in ascending order; drafts equal to the AR arg
// max are accepted up to the first mismatch, which takes the AR token; later
// drafts are left masked.
__global__ __launch_bounds__(STHREADS) void verify_scan_kernel(Args a)
{
    const int n = blockIdx.x;
    const int tid = threadIdx.x;
    // pass 1: position of the first mismatch, and the AR token there.  A position's records and its draft are
    // requested together with its mask bytes (one memory round trip instead of three); what was requested for
    // a position that is no draft is not used.
    constexpr int PRE = 8;
    int first_bad = 0x7fffffff;
    int bad_tok = 0;            // AR token at this lane's lowest mismatch
    for (int b = tid; b < a.B; b += STHREADS) {
        const size_t i = (size_t)n * a.B + b;
        const u32x4* pr = reinterpret_cast<const u32x4*>(a.ws + i * a.vsplits);
        u32x4 rec[PRE];
#pragma unroll
        for (int s = 0; s < PRE; ++s) rec[s] = s < a.vsplits ? pr[s] : u32x4{0u, 0u, 0u, 0u};
        const int d = a.draft[i];
        const bool is_draft = a.mask[i] == 1 && !(a.scaffold && a.scaffold[i]);
        if (!is_draft) continue;
        // ascending pieces: strict '>' keeps the lowest id on ties
        float M = __uint_as_float(rec[0].x);
        int arg = (int)rec[0].y;
#pragma unroll
        for (int s = 1; s < PRE; ++s)
            if (s < a.vsplits && __uint_as_float(rec[s].x) > M) { M = __uint_as_float(rec[s].x); arg = (int)rec[s].y; }
        const Partial* p = a.ws + i * a.vsplits;
        for (int s = PRE; s < a.vsplits; ++s)
            if (p[s].m > M) { M = p[s].m; arg = p[s].arg; }
        if (arg != d && b < first_bad) { first_bad = b; bad_tok = arg; }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) first_bad = min(first_bad, __shfl_xor(first_bad, off, 64));
    // pass 2: accept up to it, replace at it, leave the rest
    int count = 0;
    for (int b = tid; b < a.B; b += STHREADS) {
        const size_t i = (size_t)n * a.B + b;
        const bool is_draft = a.mask[i] == 1 && !(a.scaffold && a.scaffold[i]);
        uint8_t acc = 0;
        if (is_draft && b <= first_bad) {
            acc = (b == first_bad) ? 2 : 1;
            // (the lane that visits position first_bad met no mismatch below it: bad_tok is the token there)
            a.tokens[i] = (b == first_bad) ? bad_tok : a.draft[i];
            a.mask[i] = 0;
            ++count;
        }
        if (a.committed) a.committed[i] = acc;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) count += __shfl_xor(count, off, 64);
    if (tid == 0 && a.n_unmasked) a.n_unmasked[n] = count;
}

}  // namespace

bool make_unmask_plan(const fdd_unmask_params& p, UnmaskPlan* plan)
{
    return make_vocab_plan(p.N, p.B, p.V, p.dtype, false, plan);
}

bool make_vocab_plan(int N, int B, long long V, int dtype, bool argmax_only, UnmaskPlan* plan)
{
    struct { int N, B; long long V; int dtype; } p = {N, B, V, dtype};
    if (p.N <= 0 || p.B <= 0 || p.V <= 0) return false;
    const long long rows = (long long)p.N * p.B;
    const long long es = p.dtype == FDD_BF16 ? 2 : 4;
    long long by_size = (p.V * es) / ((argmax_only ? PIECE_KB_ARGMAX : PIECE_KB) * 1024);     // keep pieces at this size or more
    if (by_size < 1) by_size = 1;
    long long want = (8192 + rows - 1) / rows;  // enough workgroups to fill 256 CUs several times
    if (want < 1) want = 1;
    long long vs = want < by_size ? want : by_size;
    if (vs > 64) vs = 64;
    plan->vsplits = (int)vs;
    plan->ws_bytes = (size_t)rows * (size_t)vs * sizeof(Partial);
    return true;
}

hipError_t launch_unmask(const fdd_unmask_params& p, const UnmaskPlan& plan, hipStream_t s)
{
    Args a;
    a.logits = p.logits;
    a.scaffold = p.scaffold_mask;
    a.mask = p.mask;
    a.tokens = p.tokens;
    a.conf = p.confidences;
    a.n_unmasked = p.n_unmasked;
    a.committed = p.committed;
    a.ws = static_cast<Partial*>(p.workspace);
    a.draft = nullptr;
    a.rf_tk = static_cast<const u32x4*>(p.refresh_table_k);
    a.rf_tv = static_cast<const u32x4*>(p.refresh_table_v);
    a.rf_bk = static_cast<u32x4*>(p.refresh_block_k);
    a.rf_bv = static_cast<u32x4*>(p.refresh_block_v);
    a.rf_T = p.refresh_T;
    a.rf_row_vecs = p.refresh_block_k ? (int)((size_t)p.refresh_Hkv * p.refresh_D * (p.refresh_dtype == FDD_BF16 ? 2 : 4) / 16) : 0;
    a.N = p.N; a.B = p.B; a.vsplits = plan.vsplits; a.V = p.V; a.tau = p.tau;
    a.c = 0.f; a.seed_lo = 0u; a.seed_hi = 0u;
    const dim3 grid((unsigned)(plan.vsplits * p.N * p.B));
    if (p.dtype == FDD_BF16) hipLaunchKernelGGL((vocab_reduce_kernel<uint16_t, true>), grid, dim3(RTHREADS), 0, s, a);
    else hipLaunchKernelGGL((vocab_reduce_kernel<float, true>), grid, dim3(RTHREADS), 0, s, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(block_select_kernel, dim3(p.N), dim3(STHREADS), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_verify(const fdd_verify_params& p, const UnmaskPlan& plan, hipStream_t s)
{
    Args a;
    a.logits = p.ar_logits;
    a.scaffold = p.scaffold_mask;
    a.mask = p.mask;
    a.tokens = p.tokens;
    a.conf = nullptr;
    a.n_unmasked = p.n_accepted;
    a.committed = p.accepted;
    a.ws = static_cast<Partial*>(p.workspace);
    a.draft = p.draft;
    a.rf_tk = nullptr; a.rf_tv = nullptr; a.rf_bk = nullptr; a.rf_bv = nullptr; a.rf_T = 0; a.rf_row_vecs = 0;
    a.N = p.N; a.B = p.B; a.vsplits = plan.vsplits; a.V = p.V; a.tau = 0.f;
    a.c = p.temperature > 0.f ? (float)(1.4426950408889634 / (double)p.temperature) : 0.f;
    a.seed_lo = (uint32_t)p.seed;
    a.seed_hi = (uint32_t)(p.seed >> 32);
    const dim3 grid((unsigned)(plan.vsplits * p.N * p.B));
    if (p.temperature > 0.f) {
        if (p.dtype == FDD_BF16) hipLaunchKernelGGL(vocab_sample_kernel<uint16_t>, grid, dim3(RTHREADS), 0, s, a);
        else hipLaunchKernelGGL(vocab_sample_kernel<float>, grid, dim3(RTHREADS), 0, s, a);
    } else {
        // greedy verifier: step 3 of scaffold speculative decoding compares arg maxima only, so no exponentials
        if (p.dtype == FDD_BF16) hipLaunchKernelGGL((vocab_reduce_kernel<uint16_t, false>), grid, dim3(RTHREADS), 0, s, a);
        else hipLaunchKernelGGL((vocab_reduce_kernel<float, false>), grid, dim3(RTHREADS), 0, s, a);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(verify_scan_kernel, dim3(p.N), dim3(STHREADS), 0, s, a);
    return hipGetLastError();
}

}  // namespace fdd
