// Host-side driver for the sanitizer pass over the library's planner (argument checks, shape -> plan, workspace
// sizes, the weighted partition's integer functions, the plan table).  Built together with prism_api.hip with
// AddressSanitizer and UndefinedBehaviorSanitizer on the host code; the kernel launchers are stubs, so nothing
// here needs a GPU.  Exit status 0 and no sanitizer report = pass.
#include <cstdint>
#include <cstdio>
#include <cstdlib>

#include "prism_internal.h"
#include "stream_partition.h"

namespace prism {
hipError_t launch_simple_f32(const Call&) { return hipSuccess; }
hipError_t launch_simple_bf16(const Call&) { return hipSuccess; }
hipError_t launch_simple_f16(const Call&) { return hipSuccess; }
hipError_t launch_decode_16bit(const Call&, bool, int, const StreamPartition&, int, bool, const DecodeWorkspace&) { return hipSuccess; }
hipError_t launch_decode_rows_16bit(const Call&, bool, int, int, bool, const DecodeWorkspace&) { return hipSuccess; }
hipError_t launch_prefill_16bit(const Call&, bool, int, int) { return hipSuccess; }
hipError_t launch_softmax_rows_16bit(const SoftmaxCall&, bool) { return hipSuccess; }
hipError_t launch_softmax_split_16bit(const SoftmaxCall&, bool, int, const SoftmaxWorkspace&) { return hipSuccess; }
hipError_t launch_probe_stream(const void*, const void*, unsigned*, int, int, int, hipStream_t) { return hipSuccess; }
hipError_t launch_probe_units(const void*, unsigned, int, unsigned long long*, hipStream_t) { return hipSuccess; }
hipError_t launch_probe_mfma(float*, int, int, hipStream_t) { return hipSuccess; }
hipError_t launch_probe_loads(const void*, int, int, int, unsigned long long*, hipStream_t) { return hipSuccess; }
hipError_t launch_probe_linear(const void*, unsigned long long, int, unsigned*, hipStream_t) { return hipSuccess; }
hipError_t launch_softmax_simple(const SoftmaxCall&, int) { return hipSuccess; }
hipError_t launch_gqa_16bit(const AttentionCall&, bool, const AttentionPlan&, const AttentionWorkspace&) { return hipSuccess; }
hipError_t launch_gqa_simple(const AttentionCall&, int) { return hipSuccess; }
}  // namespace prism

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint64_t rnd() {  // splitmix64
    uint64_t z = (rng_state += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
static int64_t pick(const int64_t* v, int n) { return v[rnd() % (uint64_t)n]; }

#define REQUIRE(c) do { if (!(c)) { std::fprintf(stderr, "planner_driver: check failed at line %d: %s\n", __LINE__, #c); return 1; } } while (0)

int main() {
    static const int64_t rows[] = {0, 1, 2, 8, 15, 16, 17, 31, 32, 33, 63, 64, 65, 100, 128, 255, 256, 257, 511, 512, 513,
                                   1000, 4096, 20000, 65536 * 16, 0x7FFFFFFF, 0x80000000ll};
    static const int64_t deps[] = {1, 7, 8, 16, 24, 64, 72, 128, 1000, 1024, 2048, 2056, 4096, 4104, 8192, 14336, 32768,
                                   1 << 20, 1 << 24, 0x7FFFFFF8, 0x7FFFFFFF};
    static const int64_t wids[] = {0, 1, 8, 16, 64, 120, 128, 136, 1024, 4096, 4104, 7168, 11008, 14336, 18432, 20352, 33280,
                                   57344, 128256, 1 << 20, 1 << 24, 0x7FFFFFF8, 0x7FFFFFFF};
    static const int cus[] = {0, 1, 8, 32, 64, 104, 128, 228, 256, 304, 1024};
    static const int masks[] = {0, 0x0808, 0xFFFF, 0x0001, 0x8000, 0x2828};
    long plans = 0, ok_plans = 0;
    for (int it = 0; it < 60000; ++it) {
        if (it % 500 == 0) {
            REQUIRE(prism_diag_set_cu_count(cus[rnd() % 11]) == PRISM_OK);
            REQUIRE(prism_set_stream_balance(masks[rnd() % 6], (int)(rnd() % 4)) == PRISM_OK);
        }
        const prism_op_t op = (prism_op_t)(rnd() % 3);
        const prism_dtype_t dt = (prism_dtype_t)(rnd() % 3);
        const int64_t M = pick(rows, sizeof(rows) / 8), K = pick(deps, sizeof(deps) / 8), N = pick(wids, sizeof(wids) / 8);
        // a third of the calls with a forced (path, split, variant), valid or not
        if (rnd() % 3 == 0) {
            static const int variants[] = {0, 4, 8, 16, 32, 64, 104, 108, 256256, 256192, 128256, 128128, 64064, 17, 999999};
            static const int splits[] = {0, 1, 2, 3, 7, 8, 16, 33, 64, 1000, 70000};
            (void)prism_set_override((int)(rnd() % 6), splits[rnd() % 11], variants[rnd() % 15]);
        } else {
            REQUIRE(prism_set_override(0, 0, 0) == PRISM_OK);
        }
        prism_plan_t p;
        const prism_status_t st = prism_plan(op, M, K, N, dt, &p);
        REQUIRE(st >= PRISM_OK && st <= PRISM_ERR_HIP);
        ++plans;
        const uint64_t wb = prism_workspace_bytes(op, M, K, N, dt);
        if (st == PRISM_OK) {
            ++ok_plans;
            REQUIRE(wb == p.workspace_bytes);
            REQUIRE(p.split_k >= 1 && p.grid_x >= 0 && p.grid_y >= 0 && p.block >= 0 && p.block <= 1024);
            if (M > 0 && N > 0) REQUIRE(p.path >= PRISM_PATH_SIMPLE && p.path <= PRISM_PATH_ROWS && p.grid_x >= 1);
            if (p.split_k == 1) REQUIRE(p.workspace_bytes == 0);
        } else {
            REQUIRE(wb == 0);
        }
        // the entry points themselves, with pointers that are never dereferenced on the host (stub launchers)
        void* a = (void*)0x10000;
        const prism_status_t rs = (op == PRISM_OP_RMSNORM_MATMUL) ? prism_rmsnorm_matmul(a, a, a, a, M, K, N, 1e-6f, dt, nullptr)
                                  : (op == PRISM_OP_RMSNORM_GATED_MLP) ? prism_rmsnorm_gated_mlp(a, a, a, a, a, M, K, N, 1e-6f, dt, nullptr)
                                                                       : prism_softmax_matmul(a, a, a, M, K, N, dt, nullptr);
        REQUIRE(rs >= PRISM_OK && rs <= PRISM_ERR_HIP);
        if (it % 7 == 0) {
            const prism_status_t ts = prism_plan_table_set(op, M, K, N, dt, (int)(rnd() % 5), (int)(rnd() % 9), 0);
            REQUIRE(ts >= PRISM_OK && ts <= PRISM_ERR_HIP);
            if (prism_plan_table_size() > 200) REQUIRE(prism_plan_table_clear() == PRISM_OK);
        }
        if (it % 5 == 0) {
            static const int64_t bs[] = {0, 1, 2, 8, 32, 300, 65535, 65536};
            static const int64_t hs[] = {1, 17, 128, 1024, 2048, 16385, 131072, 1 << 20, 0x7FFFFFFF};
            static const int64_t ds[] = {1, 20, 64, 128, 1024, 1025};
            prism_plan_t ap;
            const int64_t B = pick(bs, 8), G = (int64_t)(rnd() % 40), H = pick(hs, 9), D = pick(ds, 6);
            const prism_status_t as = prism_attention_plan(B, G, H, D, dt, &ap);
            REQUIRE(as >= PRISM_OK && as <= PRISM_ERR_HIP);
            if (as == PRISM_OK) REQUIRE(prism_attention_workspace_bytes(B, G, H, D, dt) == ap.workspace_bytes);
        }
    }
    REQUIRE(prism_set_override(0, 0, 0) == PRISM_OK && prism_diag_set_cu_count(0) == PRISM_OK);
    // the weighted partition: every K-block of every tile dealt out exactly once, for random geometries
    for (int it = 0; it < 300; ++it) {
        const int G = 1 + (int)(rnd() % 300), kblocks = 1 + (int)(rnd() % 200), n_tiles = 1 + (int)(rnd() % 260);
        const int period = (rnd() & 1) ? 8 : 16, slow = (int)(rnd() % (1u << period));
        const int w_fast = 1 + (int)(rnd() % 8), w_slow = w_fast + (int)(rnd() % 4);
        for (int t = 0; t < n_tiles; t += 1 + (int)(rnd() % 7)) {
            long covered = 0;
            int next = 0;
            for (int wg = 0; wg < G; ++wg) {
                int32_t first = -1, count = -1;
                const prism_status_t ps = prism_stream_partition_blocks(G, kblocks, n_tiles, slow, period, w_fast, w_slow, wg, t, &first, &count);
                REQUIRE(ps == PRISM_OK || ps == PRISM_ERR_UNSUPPORTED);
                if (ps != PRISM_OK) { covered = kblocks; break; }
                REQUIRE(count >= 0 && first >= 0 && first + count <= kblocks);
                if (count > 0) { REQUIRE(first == next); next = first + count; }
                covered += count;
            }
            REQUIRE(covered == kblocks);
        }
    }
    std::printf("planner_driver: %ld plans (%ld accepted), no check failed\n", plans, ok_plans);
    return 0;
}
