// Rollout-fork bookkeeping: the private per-rollout state of forked rollouts.
//
// "Fork the KV cache N times" (paper, "Shared prefix"): the prefix is shared by
// pointer and never copied, so a fork only replicates the block-sized private
// arrays (block K/V, tokens, mask).  After an unmask step the K/V rows of the
// newly committed positions are refreshed; with no model in scope the new row
// is looked up in caller-provided tables by token id.  A finished block is
// appended to its rollout's private extension (the blocks decoded since the
// fork), which later blocks of that rollout attend to.
#include "fdd_internal.h"

namespace fdd {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void fork_kernel(int N, size_t words, int vec, const uint32_t* src, uint32_t* dst)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    const size_t i0 = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (vec) {
        const size_t n4 = words / 4;
        const u32x4* s4 = reinterpret_cast<const u32x4*>(src);
        u32x4* d4 = reinterpret_cast<u32x4*>(dst);
        for (size_t i = i0; i < n4; i += stride) {
            const u32x4 x = s4[i];
            for (int n = 0; n < N; ++n) d4[(size_t)n * n4 + i] = x;
        }
    } else {
        for (size_t i = i0; i < words; i += stride) {
            const uint32_t x = src[i];
            for (int n = 0; n < N; ++n) dst[(size_t)n * words + i] = x;
        }
    }
}

// one workgroup per block position; rows are Hkv*D elements = `row_vecs` 16-byte pieces
__global__ __launch_bounds__(256) void kv_update_kernel(int T, int row_vecs, const int32_t* tokens, const uint8_t* committed,
                                                         const u32x4* tk, const u32x4* tv, u32x4* bk, u32x4* bv)
{
    const size_t i = blockIdx.x;
    if (!committed[i]) return;
    int t = tokens[i] % T;
    if (t < 0) t += T;
    for (int c = threadIdx.x; c < row_vecs; c += blockDim.x) {
        bk[i * row_vecs + c] = tk[(size_t)t * row_vecs + c];
        bv[i * row_vecs + c] = tv[(size_t)t * row_vecs + c];
    }
}

// grid (N, chunks): rollout n's block (`block_vecs` 16-byte pieces) is copied to piece offset
// `dst0` of its extension (`ext_vecs` pieces per rollout), K and V alike
__global__ __launch_bounds__(256) void commit_kernel(size_t block_vecs, size_t ext_vecs, size_t dst0, const u32x4* bk,
                                                      const u32x4* bv, u32x4* ek, u32x4* ev)
{
    const size_t n = blockIdx.x;
    for (size_t c = (size_t)blockIdx.y * blockDim.x + threadIdx.x; c < block_vecs; c += (size_t)gridDim.y * blockDim.x) {
        ek[n * ext_vecs + dst0 + c] = bk[n * block_vecs + c];
        ev[n * ext_vecs + dst0 + c] = bv[n * block_vecs + c];
    }
}

// equal-weight mean of the N rollout trajectories, one thread per coordinate
__global__ __launch_bounds__(256) void traj_mean_kernel(int N, int P, const float* traj, float* out)
{
    const int p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= P) return;
    float acc = 0.f;
    for (int n = 0; n < N; ++n) acc += traj[(size_t)n * P + p];
    out[p] = acc / (float)N;
}

}  // namespace

hipError_t launch_traj_mean(int N, int P, const float* traj, float* out, hipStream_t s)
{
    hipLaunchKernelGGL(traj_mean_kernel, dim3((unsigned)((P + 255) / 256)), dim3(256), 0, s, N, P, traj, out);
    return hipGetLastError();
}

hipError_t launch_block_commit(const fdd_commit_params& p, hipStream_t s)
{
    const size_t es = p.dtype == FDD_BF16 ? 2 : 4;
    const size_t row_vecs = (size_t)p.Hkv * p.D * es / 16;
    const size_t block_vecs = row_vecs * p.B;
    unsigned chunks = (unsigned)((block_vecs + 255) / 256);
    if (chunks > 64) chunks = 64;
    hipLaunchKernelGGL(commit_kernel, dim3((unsigned)p.N, chunks), dim3(256), 0, s, block_vecs, row_vecs * p.ext_capacity,
                       row_vecs * p.E, static_cast<const u32x4*>(p.block_k), static_cast<const u32x4*>(p.block_v),
                       static_cast<u32x4*>(p.ext_k), static_cast<u32x4*>(p.ext_v));
    return hipGetLastError();
}

hipError_t launch_fork_block(int N, size_t bytes, const void* src, void* dst, hipStream_t s)
{
    const size_t words = bytes / 4;
    const int vec = (bytes % 16 == 0) && ((uintptr_t)src % 16 == 0) && ((uintptr_t)dst % 16 == 0);
    const size_t items = vec ? words / 4 : words;
    size_t grid = (items + 255) / 256;
    if (grid > 2048) grid = 2048;
    if (grid < 1) grid = 1;
    hipLaunchKernelGGL(fork_kernel, dim3((unsigned)grid), dim3(256), 0, s, N, words, vec,
                       static_cast<const uint32_t*>(src), static_cast<uint32_t*>(dst));
    return hipGetLastError();
}

hipError_t launch_kv_update(const fdd_kv_update_params& p, hipStream_t s)
{
    const size_t es = p.dtype == FDD_BF16 ? 2 : 4;
    const int row_vecs = (int)((size_t)p.Hkv * p.D * es / 16);
    hipLaunchKernelGGL(kv_update_kernel, dim3((unsigned)(p.N * p.B)), dim3(256), 0, s, p.T, row_vecs, p.tokens, p.committed,
                       static_cast<const u32x4*>(p.table_k), static_cast<const u32x4*>(p.table_v),
                       static_cast<u32x4*>(p.block_k), static_cast<u32x4*>(p.block_v));
    return hipGetLastError();
}

}  // namespace fdd
