// Drives the host side of the C ABI (argument checks, planning arithmetic, workspace sizes, error
// strings) under -fsanitize=address,undefined.  csrc/api.hip is compiled as it is; the kernel launchers it
// calls are replaced by the stubs below, so nothing here needs a GPU and no kernel runs.  Built and run
// by tests/test_sanitize.py.
#include <climits>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "fdd_internal.h"

namespace fdd {
static int g_launches = 0;
hipError_t launch_attn_bf16(const fdd_attn_params&, const AttnPlan&, float, hipStream_t, hipEvent_t) { ++g_launches; return hipSuccess; }
hipError_t launch_prefix_pack(const void*, int, int, int, void*, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_attn_f32(const fdd_attn_params&, const AttnPlan&, float, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_attn_combine(const fdd_attn_params&, const AttnPlan&, float, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_attn_merge_bf16(const fdd_attn_params&, const AttnPlan&, float, hipStream_t) { ++g_launches; return hipSuccess; }
bool make_unmask_plan(const fdd_unmask_params& p, UnmaskPlan* plan) { return make_vocab_plan(p.N, p.B, p.V, p.dtype, false, plan); }
bool make_vocab_plan(int N, int B, long long V, int, bool, UnmaskPlan* plan)
{
    if (N <= 0 || B <= 0 || V <= 0) return false;
    plan->vsplits = 2;
    plan->ws_bytes = (size_t)N * B * 2 * 16;
    return true;
}
hipError_t launch_unmask(const fdd_unmask_params&, const UnmaskPlan&, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_verify(const fdd_verify_params&, const UnmaskPlan&, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_fork_block(int, size_t, const void*, void*, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_kv_update(const fdd_kv_update_params&, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_block_commit(const fdd_commit_params&, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_traj_mean(int, int, const float*, float*, hipStream_t) { ++g_launches; return hipSuccess; }
}  // namespace fdd

static int fails = 0;
#define EXPECT(cond) do { if (!(cond)) { std::fprintf(stderr, "line %d: %s\n", __LINE__, #cond); ++fails; } } while (0)

// Every pointer is a fake, suitably aligned address: the stubs never touch them.
static void* fake(size_t k) { return reinterpret_cast<void*>((uintptr_t)0x10000000 + 0x1000 * k); }

static fdd_attn_params attn(int N, int B, int L, int Hq, int Hkv, int D, int dtype)
{
    fdd_attn_params p;
    std::memset(&p, 0, sizeof p);
    p.N = N; p.B = B; p.L = L; p.Hq = Hq; p.Hkv = Hkv; p.D = D; p.dtype = dtype;
    p.q = fake(1); p.prefix_k = fake(2); p.prefix_v = fake(3); p.block_k = fake(4); p.block_v = fake(5); p.out = fake(6);
    return p;
}

int main()
{
    // planning arithmetic over a sweep of shapes, including the extremes the checks let through
    const int Ns[] = {1, 2, 3, 8, 16, 64, 1000}, Bs[] = {1, 7, 32, 64, 100}, Ls[] = {0, 1, 63, 64, 65, 2048, 16384, 1000000};
    const int heads[][2] = {{4, 1}, {28, 4}, {8, 8}, {64, 8}};
    long planned = 0;
    for (int dtype = 0; dtype < 2; ++dtype)
        for (int N : Ns) for (int B : Bs) for (int L : Ls) for (auto& h : heads) for (int D : {64, 128})
            for (int splits : {0, 1, 5, 64}) for (int E : {0, 70}) {
                fdd_attn_params p = attn(N, B, L, h[0], h[1], D, dtype);
                p.splits = splits; p.E = E; p.ext_capacity = E ? 128 : 0; p.ext_k = fake(7); p.ext_v = fake(8);
                const size_t need = fdd_block_attn_workspace(&p);
                std::vector<char> dummy;     // (sizes only: the workspace pointer is a fake as well)
                p.workspace = need ? fake(9) : nullptr; p.workspace_bytes = need;
                const fdd_status st = fdd_block_attn(&p);
                EXPECT(st == FDD_OK || st == FDD_ERR_SHAPE);
                if (st == FDD_OK) ++planned;
                if (need > 0) {
                    p.workspace_bytes = need - 1;
                    EXPECT(fdd_block_attn(&p) == FDD_ERR_WORKSPACE);
                }
            }
    EXPECT(planned > 1000);
    // lists of query positions, batches, packed prefixes
    {
        fdd_attn_params p = attn(16, 64, 16384, 28, 4, 128, FDD_BF16);
        p.prefix_v_packed = fake(10);
        p.q_positions = reinterpret_cast<const int32_t*>(fake(11)); p.n_q_positions = 720;
        size_t need = fdd_block_attn_workspace(&p);
        p.workspace = fake(12); p.workspace_bytes = need;
        EXPECT(fdd_block_attn(&p) == FDD_OK);
        p.n_q_positions = 16 * 64 + 1;
        EXPECT(fdd_block_attn(&p) == FDD_ERR_SHAPE);
        p.n_q_positions = 0; p.batch = 28; p.q_batch_stride = 1;
        EXPECT(fdd_block_attn(&p) == FDD_ERR_SHAPE);
        p.batch = 70000;
        EXPECT(fdd_block_attn(&p) == FDD_ERR_SHAPE);
    }
    // argument errors: every code, and the message is always terminated
    {
        EXPECT(fdd_block_attn(nullptr) == FDD_ERR_NULL);
        fdd_attn_params p = attn(INT_MAX, INT_MAX, INT_MAX, 28, 4, 128, FDD_BF16);
        EXPECT(fdd_block_attn(&p) == FDD_ERR_SHAPE);
        EXPECT(fdd_block_attn_workspace(&p) == 0);
        p = attn(1, 1, 1, 7, 2, 128, FDD_BF16);
        EXPECT(fdd_block_attn(&p) == FDD_ERR_SHAPE);
        p = attn(1, 1, 1, 4, 2, 96, FDD_BF16);
        EXPECT(fdd_block_attn(&p) == FDD_ERR_UNSUPPORTED);
        p = attn(1, 1, 1, 4, 2, 64, 7);
        EXPECT(fdd_block_attn(&p) == FDD_ERR_DTYPE);
        p = attn(1, 1, 1, 4, 2, 64, FDD_F32);
        p.q = nullptr;
        EXPECT(fdd_block_attn(&p) == FDD_ERR_NULL);
        EXPECT(std::strlen(fdd_last_error()) > 0 && std::strlen(fdd_last_error()) < 384);
        EXPECT(fdd_prefix_pack(fake(1), INT_MAX, INT_MAX, 128, FDD_BF16, fake(2), 0, nullptr) == FDD_ERR_SHAPE);
        EXPECT(fdd_prefix_pack_bytes(INT_MAX, 4, 128, FDD_BF16) > 0);
        EXPECT(fdd_prefix_pack(fake(1), 4096, 4, 128, FDD_BF16, fake(2), 16, nullptr) == FDD_ERR_WORKSPACE);
    }
    // unmask / verify / bookkeeping entry points
    {
        fdd_unmask_params u;
        std::memset(&u, 0, sizeof u);
        u.N = 16; u.B = 64; u.V = 152064; u.dtype = FDD_BF16; u.tau = 0.9f;
        u.logits = fake(1); u.mask = reinterpret_cast<uint8_t*>(fake(2)); u.tokens = reinterpret_cast<int32_t*>(fake(3));
        u.confidences = reinterpret_cast<float*>(fake(4));
        EXPECT(fdd_unmask_step(&u) == FDD_ERR_WORKSPACE);
        u.workspace = fake(5); u.workspace_bytes = fdd_unmask_workspace(&u);
        EXPECT(fdd_unmask_step(&u) == FDD_OK);
        u.V = (1ll << 31);
        EXPECT(fdd_unmask_step(&u) == FDD_ERR_SHAPE && fdd_unmask_workspace(&u) == 0);
        u.V = 10; u.N = INT_MAX; u.B = INT_MAX;
        EXPECT(fdd_unmask_step(&u) == FDD_ERR_SHAPE);
        fdd_verify_params v;
        std::memset(&v, 0, sizeof v);
        v.N = 4; v.B = 8; v.V = 1000; v.dtype = FDD_F32; v.temperature = -1.f;
        EXPECT(fdd_verify_step(&v) == FDD_ERR_UNSUPPORTED);
        v.temperature = 0.5f;
        EXPECT(fdd_verify_step(&v) == FDD_ERR_NULL);
        EXPECT(fdd_fork_block(4, 1024, fake(1), fake(1), nullptr) == FDD_ERR_UNSUPPORTED);
        EXPECT(fdd_fork_block(4, 1024, fake(1), fake(20), nullptr) == FDD_OK);
        EXPECT(fdd_fork_block(INT_MAX, (size_t)-4, fake(1), fake(20), nullptr) != FDD_OK);
        fdd_commit_params c;
        std::memset(&c, 0, sizeof c);
        c.N = 2; c.B = 32; c.Hkv = 4; c.D = 128; c.dtype = FDD_BF16; c.E = INT_MAX; c.ext_capacity = INT_MAX;
        c.block_k = fake(1); c.block_v = fake(2); c.ext_k = fake(3); c.ext_v = fake(4);
        EXPECT(fdd_block_commit(&c) == FDD_ERR_SHAPE);
        EXPECT(fdd_traj_mean(0, 5, reinterpret_cast<const float*>(fake(1)), reinterpret_cast<float*>(fake(2)), nullptr) == FDD_ERR_SHAPE);
        fdd_kv_update_params k;
        std::memset(&k, 0, sizeof k);
        EXPECT(fdd_block_kv_update(&k) == FDD_ERR_SHAPE);
    }
    EXPECT(fdd::g_launches > 0);
    if (fails) return 1;
    std::puts("ABI host sanitizer run: ok");
    return 0;
}
