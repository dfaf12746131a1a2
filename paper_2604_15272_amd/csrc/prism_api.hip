// C ABI of the library: argument checks, shape -> kernel dispatch, workspace bookkeeping.
#include <atomic>
#include <algorithm>
#include <cmath>
#include <cstring>
#include <mutex>

#include "prism_internal.h"
#include "stream_partition.h"

// Split-K scratch of prism_rmsnorm_matmul_static: the same layout as a registered workspace (arrival counters,
// partial sums of squares, partial products), held by every device the library runs on until the process ends.
// In host code this name is a stand-in, not a device address: the address is asked for once per device
// (static_scratch below) and only that pointer is handed to kernels.
static __device__ __align__(256) unsigned char scratch[PRISM_STATIC_SCRATCH_BYTES];

namespace prism {
namespace {

__global__ void clear_words_kernel(unsigned* p, unsigned n) {
    const unsigned i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

constexpr int kMaxDevices = 64;
constexpr uint64_t kTwoGiB = 0x7FFFFFFFull;

struct Override {
    std::atomic<int32_t> path{0}, split_k{0}, variant{0};
};
Override g_override;

// Address slots that stream slowly, and what the 16-row decode kernel does about them.
// Measured on MI355X with per-workgroup time stamps: when the row pitch of W is a multiple of 2 KiB, the stripe of
// W a workgroup streams keeps bits 7-10 of its byte addresses for all rows (which 128 bytes of every 2 KiB: its
// unit), and the stripes in units 3 and 11 arrive 40 % later than the others (44 us against 32 us for
// 128-byte-wide stripes of 2 x W[4096,14336]; 256-byte-wide stripes that contain them: 37 us against 30 us),
// whichever XCD reads them and wherever W starts; a row pitch of 225 x 256 bytes, which takes every workgroup
// through all units, ends all stripes at 32 us.
//  - g_slow_units: bit u set = unit u is slow.
//  - g_stream_mode bit 0: the two-pass weighted partition of stream_partition.h for 129 to 159 column tiles (off:
//    a grid of three K-slices per tile is faster there, see make_plan_with); bit 1: in that partition, 256-byte
//    tiles that contain a slow unit weigh 5 : 4.
// Gated calls with at most 16 rows use the packed tile (64 output columns: 128-byte stripes of W1 and of W2) with
// more K-slices for the tiles in slow units when that fits the CUs: 42.1 -> 40.7 us on X[8,4096], 2 x W[4096,14336].
// No unit is taken to be slow until the caller says so (prism_set_stream_balance; the Python package's tuner
// measures the sixteen units on the machine at hand): which units are slow is a property of a machine, not of the
// method.
std::atomic<int32_t> g_slow_units{0}, g_stream_mode{0};

struct Workspace {
    void* ptr;
    uint64_t bytes;
};
Workspace g_workspace[kMaxDevices];  // indexed by HIP device ordinal: the workspace of calls on any stream
// Workspaces registered for one stream each (prism_set_stream_workspace): calls on that stream use theirs, so that
// two streams can run split-K calls at the same time without sharing arrival counters.
struct StreamWorkspace {
    int dev;
    hipStream_t stream;
    Workspace ws;
};
constexpr int kMaxStreamWorkspaces = 32;
StreamWorkspace g_stream_ws[kMaxStreamWorkspaces];
int g_stream_ws_count = 0;
std::mutex g_ws_mutex;

// The workspace a call on `stream` of the current device uses.
prism_status_t workspace_for(hipStream_t stream, Workspace* out) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return PRISM_ERR_HIP;
    if (dev < 0 || dev >= kMaxDevices) return PRISM_ERR_WORKSPACE;
    std::lock_guard<std::mutex> lock(g_ws_mutex);
    for (int i = 0; i < g_stream_ws_count; ++i)
        if (g_stream_ws[i].dev == dev && g_stream_ws[i].stream == stream) {
            *out = g_stream_ws[i].ws;
            return PRISM_OK;
        }
    *out = g_workspace[dev];
    return PRISM_OK;
}

uint64_t round_up(uint64_t v, uint64_t a) { return (v + a - 1) / a * a; }

// Compute units of the device the plans are made for: the current device's count, asked once per process (all
// devices of a node are alike); 256, an MI355X in its default partition mode, where no device can be asked (the
// planner also runs on hosts without a GPU).  prism_diag_set_cu_count replaces it for tests.
constexpr int kDefaultCus = 256;
std::atomic<int> g_cus{0}, g_cus_forced{0};

int64_t cu_count() {
    if (const int f = g_cus_forced.load(std::memory_order_relaxed); f > 0) return f;
    int v = g_cus.load(std::memory_order_relaxed);
    if (v > 0) return v;
    int dev = 0, n = 0;
    v = (hipGetDevice(&dev) == hipSuccess &&
         hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0) ? n : kDefaultCus;
    (void)hipGetLastError();  // a host without a device: the failed query is not this library's error to report later
    g_cus.store(v, std::memory_order_relaxed);
    return v;
}

// Address of `scratch` on the current device, looked up on the first call there.  That call also clears the arrival
// counters with a small kernel on the caller's stream (a kernel, not a memset, so that a caller who is recording a
// graph records something that replays correctly); afterwards every kernel leaves them at zero.
void* g_scratch_ptr[kMaxDevices];
std::mutex g_scratch_mutex;

prism_status_t static_scratch(hipStream_t stream, Workspace* out) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return PRISM_ERR_HIP;
    if (dev < 0 || dev >= kMaxDevices) return PRISM_ERR_WORKSPACE;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return PRISM_ERR_HIP;
        constexpr unsigned words = PRISM_WORKSPACE_HEADER_BYTES / 4;
        hipLaunchKernelGGL(clear_words_kernel, dim3(words / 256), dim3(256), 0, stream, (unsigned*)p, words);
        if (hipGetLastError() != hipSuccess) return PRISM_ERR_HIP;
        g_scratch_ptr[dev] = p;
    }
    *out = Workspace{g_scratch_ptr[dev], PRISM_STATIC_SCRATCH_BYTES};
    return PRISM_OK;
}

struct Plan {
    prism_plan_t pub;
    int waves;          // decode: wavefronts per workgroup
    int row_groups;     // decode: 16-row groups per workgroup (1: the 16-row kernel)
    bool xlds;          // decode, several row groups: X through LDS
    bool packed;        // decode, 16-row kernel, gated: 64 output columns per tile, both matrices in one MFMA tile
    StreamPartition sp; // decode, 16-row kernel: weighted partition (G = 0: plain grid); slow = the slots, not yet
                        // rotated to the address of W
    int base_split;     // decode, packed and balanced: K-slices of a tile outside the slow units (the grid to fall
                        // back to when W is not aligned to its units)
    uint64_t ss_bytes;  // decode: bytes of the partial sums of squares (rounded)
};

bool vector16_ok(int64_t K, int64_t N) { return K % 8 == 0 && N % 8 == 0; }
bool dtype_known(prism_dtype_t d) { return d == PRISM_F32 || d == PRISM_BF16 || d == PRISM_F16; }

// Prefill tile choice: fewest "rounds" of 256 workgroups, weighted by how well a tile shape feeds
// the matrix cores (bigger tiles re-read less from LDS per MFMA).
struct Tile {
    int bm, bn;
    double eff;
};

void choose_prefill_tile(bool gated, int64_t M, int64_t N, int variant, int* bm, int* bn) {
    // (efficiencies from every tile forced on 162 shapes of 513 to 4096 rows, plain and gated: the choice is the
    // fastest tile or within 6 % of it; with 0.85 for the gated 128 x 256 tile it lost 6 % on average and up to 26 %)
    static const Tile plain[] = {{256, 256, 1.0}, {256, 192, 0.9}, {256, 128, 0.75}, {128, 128, 0.7}, {64, 64, 0.35}};
    static const Tile gate[] = {{256, 256, 1.0}, {128, 256, 0.55}, {128, 128, 0.65}};
    const Tile* t = gated ? gate : plain;
    const int nt = gated ? 3 : 5;
    if (variant > 0) {
        *bm = variant / 1000;
        *bn = variant % 1000;
        return;
    }
    double best = 1e300;
    for (int i = 0; i < nt; ++i) {
        const int cw = gated ? t[i].bn / 2 : t[i].bn;
        const double tiles = (double)((M + t[i].bm - 1) / t[i].bm) * (double)((N + cw - 1) / cw);
        const double rounds = std::ceil(tiles / (double)cu_count());
        const double cost = rounds * t[i].bm * t[i].bn / t[i].eff;
        if (cost < best) {
            best = cost;
            *bm = t[i].bm;
            *bn = t[i].bn;
        }
    }
}

// More than 16 rows: which kernel family takes the call.  Returns the 16-row groups per workgroup of the decode
// path's multi-row kernel (2 or 4: 32 or 64 rows), or 0 if the tiled prefill kernel is the better choice.
//
// The choice is made by a small time model of the three candidates, whose constants were measured on MI355X
// (bf16, 96 shapes: 40 to 512 rows against K x N from 2048 x 8192 to 14336 x 4096, plain and gated, each forced
// onto 32 rows, 64 rows and the prefill kernel): the model's pick is within 1.1 % of the best of the three on
// average and within 10 % on every shape (the fixed rules it replaces: 4.3 % and 72 %).  Checked again on a second
// grid (17 to 512 rows against ten K x N from 1024 x 4096 to 8192 x 28672, plain and gated, 300 calls), which the
// HBM terms and the second-round factor come from: 0.2 % on average, 16 % at worst (2.4 % / 40 % for gated calls
// before them).
//   multi-row kernel, RG row groups, S K-slices, z row blocks, all times in microseconds:
//     loop      = ceil(kblocks / S) x c x rounds (x 1.1 from the second round on),  c = 0.22 / 0.31 per K-block for
//                 32 / 64 rows of one matrix, 0.33 / 0.60 for two (per compute unit a K-block costs its MFMAs, its
//                 vector work and 8 to 12 KiB through the L1, and they do not overlap); rounds = ceil(workgroups /
//                 compute units);
//                 never less than streaming W at 6 TB/s: once, or once per row block when W is beyond 128 MB
//     reduction = 0.5 x RG x matrices (LDS)
//     exchange  = 2.5 + S x RG x matrices / 8 when S > 1 (three dependent round trips, then the last arrival
//                 pulls S partial tiles through one compute unit)
//     launch    = 1.5
//   prefill kernel: K steps x (1.5 / 2.0 for 256-row tiles of one / two matrices, 1.25 for 256 x 128, 0.88 to 1.2 for
//     128-row tiles, 0.93 for 64 x 64) x 1 if every tile has a compute unit, x 1.2 for up to two 128-row tiles per
//     unit, else the rounds; + 3.  (A K step of that kernel has a floor of about a microsecond whatever the tile.)
struct RowsEstimate {
    double us;
    int64_t S;
};

RowsEstimate rows_estimate(int rg, bool gated, int64_t M, int64_t K, int64_t N, int64_t cus) {
    const int G = gated ? 2 : 1;
    const int64_t n_tiles = (N + kDecodeTileN - 1) / kDecodeTileN, kblocks = (K + kDecodeKBlock - 1) / kDecodeKBlock;
    const int64_t z = (M + 16 * rg - 1) / (16 * rg), wgs1 = n_tiles * z;
    int64_t S = wgs1 <= cus ? cus / wgs1 : 1;
    S = std::max<int64_t>(1, std::min<int64_t>(S, std::max<int64_t>(1, kblocks / 8)));
    const double c = gated ? (rg == 2 ? 0.33 : 0.60) : (rg == 2 ? 0.22 : 0.31);
    const int64_t rounds = (wgs1 * S + cus - 1) / cus;
    double loop = (double)((kblocks + S - 1) / S) * c * (double)rounds * (rounds >= 2 ? 1.1 : 1.0);
    // Never faster than W streams from HBM; weights too large for the last-level cache to keep between the row
    // blocks of a tile (256 MB; 128 MB taken) stream once per row block (gated 4096 x 14336, 48 rows as 2 x 32:
    // 58.7 us against 47.3 us for 32 rows; 8192 x 28672: 321 against 156 us).
    const double w_bytes = 2.0 * (double)K * (double)N * G;
    loop = std::max(loop, w_bytes / 6.0e6 * (w_bytes > 128.0e6 ? (double)z : 1.0));
    double us = loop + 0.5 * rg * G + 1.5;
    if (S > 1) us += 2.5 + (double)(S * rg * G) / 8.0;
    return RowsEstimate{us, S};
}

double prefill_estimate(bool gated, int64_t M, int64_t K, int64_t N, int64_t cus) {
    struct T {
        int bm, bn;
        double step;
    };
    static const T plain[] = {{256, 256, 1.5}, {256, 192, 1.5}, {256, 128, 1.25}, {128, 128, 0.88}, {64, 64, 0.93}};
    static const T gate[] = {{256, 256, 2.0}, {128, 256, 1.2}, {128, 128, 0.90}};
    // The tile the call would get (choose_prefill_tile), not the best of all: the estimate is of what would run.
    int bm = 0, bn = 0;
    choose_prefill_tile(gated, M, N, 0, &bm, &bn);
    double step = 1.5;
    for (const T& t : plain)
        if (!gated && t.bm == bm && t.bn == bn) step = t.step;
    for (const T& t : gate)
        if (gated && t.bm == bm && t.bn == bn) step = t.step;
    const int64_t KT = (K + 63) / 64;
    const int64_t cw = gated ? bn / 2 : bn;
    const int64_t tiles = ((M + bm - 1) / bm) * ((N + cw - 1) / cw);
    const bool shares_cu = bm <= 128 && bn <= 128;
    const double f = tiles <= cus ? 1.0 : ((shares_cu && tiles <= 2 * cus) ? 1.2 : (double)((tiles + cus - 1) / cus));
    // (the tiled kernel streams W from HBM at about 5 TB/s at best: gated 17 x 8192 x 28672 193 us)
    return std::max((double)KT * step * f, 2.0 * (double)K * (double)N * (gated ? 2 : 1) / 5.0e6) + 3.0;
}

int decode_row_groups(bool gated, int64_t M, int64_t K, int64_t N) {
    const int64_t n_tiles = (N + kDecodeTileN - 1) / kDecodeTileN;
    const int64_t z32 = (M + 31) / 32;
    const int64_t cus = cu_count();
    // Two weight matrices and at most one K-step of the tiled kernel: nothing to tile, and with so few products
    // per sum the tiled kernel's single rounding of g * w shows in the far tail of the outputs (2.1e-2 to 2.7e-2
    // seen in bf16 against a bar of 2e-2); the decode kernels carry x * g in two parts.
    if (gated && K <= 64 && z32 <= 65535 && n_tiles * z32 <= kMaxTickets) return 2;
    if (M > kDecodeRowsMax) return 0;
    const RowsEstimate r32 = rows_estimate(2, gated, M, K, N, cus), r64 = rows_estimate(4, gated, M, K, N, cus);
    const double pf = prefill_estimate(gated, M, K, N, cus);
    // the arrival counters of a split call: one per (column tile, row block)
    const bool ok32 = r32.S == 1 || n_tiles * z32 <= kMaxTickets;
    const bool ok64 = r64.S == 1 || n_tiles * ((M + 63) / 64) <= kMaxTickets;
    const double t32 = ok32 ? r32.us : 1e300, t64 = ok64 ? r64.us : 1e300;
    if (pf <= t32 && pf <= t64) return 0;
    return t32 <= t64 ? 2 : 4;
}

bool prefill_tile_known(bool gated, int bm, int bn) {
    if (gated) return (bm == 256 && bn == 256) || (bm == 128 && bn == 256) || (bm == 128 && bn == 128);
    return (bm == 256 && bn == 256) || (bm == 256 && bn == 192) || (bm == 256 && bn == 128) || (bm == 128 && bn == 128) ||
           (bm == 64 && bn == 64);
}

// A parameter assignment (paper Section 5, "parameter instantiation"): kernel family, split-K
// factor and tile / wavefront variant; 0 = let the built-in heuristic choose.
struct Choice {
    int path, split_k, variant;
};

// Per-shape assignments installed by a tuner.  A fixed table, searched linearly: tuned shapes are few.
struct TableEntry {
    int32_t op, dtype;
    int64_t M, K, N;
    Choice c;
};
constexpr int kTableCapacity = 256;
TableEntry g_table[kTableCapacity];
int g_table_size = 0;
std::mutex g_table_mutex;

// The process-wide override wins; then an entry of the plan table for exactly this call; then the heuristic.
Choice resolve_choice(prism_op_t op, int64_t M, int64_t K, int64_t N, prism_dtype_t dtype) {
    const Choice o{g_override.path.load(), g_override.split_k.load(), g_override.variant.load()};
    if (o.path != 0 || o.split_k != 0 || o.variant != 0) return o;
    std::lock_guard<std::mutex> lock(g_table_mutex);
    for (int i = 0; i < g_table_size; ++i) {
        const TableEntry& e = g_table[i];
        if (e.op == (int32_t)op && e.dtype == (int32_t)dtype && e.M == M && e.K == K && e.N == N) return e.c;
    }
    return Choice{0, 0, 0};
}

// Softmax -> MatMul: the matrix-core kernels for 16-bit storage with K and N multiples of 8 (variant 16: 16 rows
// per workgroup over the whole of K; variant 32: 32 rows and one of split_k K-slices), else the plain one.
prism_status_t make_softmax_plan(int64_t M, int64_t K, int64_t N, prism_dtype_t dtype, Choice choice, Plan* out) {
    std::memset(out, 0, sizeof(*out));
    prism_plan_t& p = out->pub;
    p.split_k = 1;
    if (choice.path != PRISM_PATH_AUTO && choice.path != PRISM_PATH_SIMPLE && choice.path != PRISM_PATH_ROWS)
        return PRISM_ERR_UNSUPPORTED;
    if (choice.variant != 0 && choice.variant != 16 && choice.variant != 32) return PRISM_ERR_UNSUPPORTED;
    if (M == 0 || N == 0) return PRISM_OK;
    const bool fast_ok = dtype != PRISM_F32 && vector16_ok(K, N) && (uint64_t)K * N * 2 < kTwoGiB &&
                         K <= (1 << 24) && (M + kSoftmaxRows - 1) / kSoftmaxRows <= 65535;
    int path = choice.path;
    if (path == PRISM_PATH_AUTO) path = fast_ok ? PRISM_PATH_ROWS : PRISM_PATH_SIMPLE;
    if (path == PRISM_PATH_ROWS && !fast_ok) return PRISM_ERR_UNSUPPORTED;
    p.path = path;
    if (path == PRISM_PATH_SIMPLE) {
        if (choice.split_k > 1 || choice.variant != 0) return PRISM_ERR_UNSUPPORTED;
        p.block = 256;
        p.tile_m = 8;
        p.tile_n = 256;
        p.grid_x = (int32_t)((N + 255) / 256);
        const int64_t gy = (M + 7) / 8;
        if (gy > 65535) return PRISM_ERR_UNSUPPORTED;
        p.grid_y = (int32_t)gy;
        return PRISM_OK;
    }
    const int64_t n_tiles = (N + kSoftmaxTileN - 1) / kSoftmaxTileN;
    const int64_t kblocks = (K + 31) / 32;
    const int64_t rb32 = (M + kSoftmaxSplitRows - 1) / kSoftmaxSplitRows;
    const int64_t rb16 = (M + kSoftmaxRows - 1) / kSoftmaxRows;
    int64_t S = choice.split_k;
    int variant = choice.variant;
    if (S <= 0 && variant == 16) S = 1;
    if (S <= 0) {
        // A time model of the candidates, in microseconds, with constants measured on MI355X (K-blocks of 32, eight
        // wavefronts per workgroup, so a wavefront makes kblocks / 8 trips):
        //   16 rows, whole K:   5 + rounds x trips x (0.60 + 0.35 fill)
        //   32 rows, S slices:  7.5 + rounds x trips x (0.80 + 0.60 fill) + [S > 1] (0.5 + 0.9 log2 S (1 + fill))
        // fill = workgroups / compute units, at most 1; rounds = workgroups over compute units, rounded up.  The
        // 32-row kernel reads half the W per row (it wins over several rounds) and can cut a deep K into slices
        // (it wins when there are few workgroups); handing partials across slices costs the last term.
        const double cus = (double)cu_count();
        auto rows16 = [&]() {
            const double w = (double)(n_tiles * rb16), fill = std::min(1.0, w / cus);
            return 5.0 + std::ceil(w / cus) * std::ceil((double)kblocks / 8.0) * (0.60 + 0.35 * fill);
        };
        auto rows32 = [&](int64_t s) {
            const double w = (double)(n_tiles * rb32 * s), fill = std::min(1.0, w / cus);
            const double trips = std::ceil(std::ceil((double)kblocks / (double)s) / 8.0);
            double t = 7.5 + std::ceil(w / cus) * trips * (0.80 + 0.60 * fill);
            if (s > 1) t += 0.5 + 0.9 * std::log2((double)s) * (1.0 + fill);
            return t;
        };
        auto slices_ok = [&](int64_t s) {
            if (s == 1) return true;
            return s <= kblocks && n_tiles * rb32 <= kMaxTickets && (uint64_t)s * M * N * 4 < kTwoGiB;
        };
        double best = (variant == 32 || rb32 > 65535) ? 1e300 : rows16();
        int64_t best_s = 1;
        int best_v = 16;
        if (variant != 16 && rb32 <= 65535) {
            for (int64_t s = 1; s <= kSoftmaxMaxSplits; s *= 2) {
                if (s > 1 && kblocks / s < 8) break;  // a slice keeps at least one trip of every wavefront
                if (!slices_ok(s)) continue;
                const double t = rows32(s);
                if (t < best) {
                    best = t;
                    best_s = s;
                    best_v = 32;
                }
            }
        }
        S = best_s;
        if (variant == 0) variant = best_v;
    }
    if (S > kblocks) S = kblocks;
    if (variant == 0) variant = 32;
    if (variant == 16 && S != 1) return PRISM_ERR_UNSUPPORTED;
    if (S > kSoftmaxMaxSplits) return PRISM_ERR_UNSUPPORTED;
    p.block = 512;
    p.tile_n = kSoftmaxTileN;
    p.grid_x = (int32_t)n_tiles;
    p.split_k = (int32_t)S;
    if (variant == 16) {
        p.tile_m = kSoftmaxRows;
        p.grid_y = (int32_t)((M + kSoftmaxRows - 1) / kSoftmaxRows);
        return PRISM_OK;
    }
    if (rb32 > 65535 || (S > 1 && n_tiles * rb32 > kMaxTickets)) return PRISM_ERR_UNSUPPORTED;
    if (S > 1 && (uint64_t)S * M * N * 4 >= kTwoGiB) return PRISM_ERR_UNSUPPORTED;  // 31-bit offsets into the partials
    p.tile_m = kSoftmaxSplitRows;
    p.grid_y = (int32_t)S;
    p.grid_z = (int32_t)rb32;
    if (S > 1) {
        out->ss_bytes = round_up((uint64_t)n_tiles * rb32 * S * kSoftmaxSplitRows * 2 * 4, 256);
        p.workspace_bytes = PRISM_WORKSPACE_HEADER_BYTES + out->ss_bytes + (uint64_t)S * M * N * 4;
    }
    return PRISM_OK;
}

prism_status_t make_plan_with(prism_op_t op, int64_t M, int64_t K, int64_t N, prism_dtype_t dtype, Choice choice,
                              Plan* out) {
    if (op != PRISM_OP_RMSNORM_MATMUL && op != PRISM_OP_RMSNORM_GATED_MLP && op != PRISM_OP_SOFTMAX_MATMUL)
        return PRISM_ERR_UNSUPPORTED;
    if (!dtype_known(dtype)) return PRISM_ERR_UNSUPPORTED;
    if (M < 0 || N < 0 || K <= 0) return PRISM_ERR_INVALID_ARG;
    if (M > 0x7FFFFFFF || N > 0x7FFFFFFF || K > 0x7FFFFFFF) return PRISM_ERR_UNSUPPORTED;
    if (op == PRISM_OP_SOFTMAX_MATMUL) return make_softmax_plan(M, K, N, dtype, choice, out);
    const bool gated = op == PRISM_OP_RMSNORM_GATED_MLP;
    const int forced = choice.path;
    const int forced_split = choice.split_k;
    const int variant = choice.variant;
    std::memset(out, 0, sizeof(*out));
    prism_plan_t& p = out->pub;
    p.split_k = 1;

    int path = forced;
    if (path < PRISM_PATH_AUTO || path > PRISM_PATH_PREFILL) return PRISM_ERR_UNSUPPORTED;  // PRISM_PATH_ROWS is softmax only
    if (M == 0 || N == 0) return PRISM_OK;  // empty problem: nothing is launched
    const bool fast_ok = dtype != PRISM_F32 && vector16_ok(K, N);
    if (path == PRISM_PATH_AUTO) {
        if (!fast_ok) path = PRISM_PATH_SIMPLE;
        else path = (M <= kDecodeMaxRows || decode_row_groups(gated, M, K, N) > 0) ? PRISM_PATH_DECODE : PRISM_PATH_PREFILL;
        // Shapes whose byte offsets do not fit the 32-bit buffer addressing fall back.
        if (path == PRISM_PATH_PREFILL && (uint64_t)K * N * 2 >= kTwoGiB) path = PRISM_PATH_SIMPLE;
        if (path == PRISM_PATH_DECODE && (uint64_t)M * K * 2 >= kTwoGiB) path = PRISM_PATH_SIMPLE;
    }
    p.path = path;

    if (path == PRISM_PATH_SIMPLE) {
        p.tile_m = 8;
        p.tile_n = 256;
        p.grid_x = (int32_t)((N + 255) / 256);
        p.grid_y = (int32_t)((M + 7) / 8);
        p.block = 256;
        if (p.grid_y > 65535) return PRISM_ERR_UNSUPPORTED;
        return PRISM_OK;
    }
    if (!fast_ok) return PRISM_ERR_UNSUPPORTED;

    if (path == PRISM_PATH_DECODE) {
        if ((uint64_t)M * K * 2 >= kTwoGiB) return PRISM_ERR_UNSUPPORTED;
        // Variant: 4, 8 or 16 wavefronts for at most 16 rows; 32 or 64 rows per workgroup for more.
        int waves = 8, row_groups = 1;
        bool packed = false, xlds = false;
        if (M <= kDecodeMaxRows) {
            // Variants 4, 8, 16: wavefronts per workgroup; 104, 108 (gated only): the same with the packed tile.
            int v = variant;
            if (v >= 100) {
                if (!gated) return PRISM_ERR_UNSUPPORTED;
                packed = true;
                v -= 100;
                if (v != 4 && v != 8) return PRISM_ERR_UNSUPPORTED;
            }
            if (v > 0) waves = v;
            if (waves != 4 && waves != 8 && waves != 16) return PRISM_ERR_UNSUPPORTED;
        } else {
            // Every 16-row group reuses the B operands built from W: 64 rows per workgroup unless the
            // registers (gated: two weight matrices) or the row count say 32.
            row_groups = decode_row_groups(gated, M, K, N);
            if (row_groups == 0) row_groups = 4;  // forced onto a shape the heuristic leaves to prefill
            // Variants 32 / 64: rows per workgroup, X loaded straight into operand registers; 36 / 68 (one weight
            // matrix only): the same with X through LDS (wide loads of four K-blocks at a time).  Not forced: the
            // second form where a slice gives every wavefront at least two of those super-blocks.
            if (variant == 32 || variant == 64) row_groups = variant / 16;
            else if (variant == 36 || variant == 68) {
                if (gated) return PRISM_ERR_UNSUPPORTED;
                row_groups = (variant - 4) / 16;
                xlds = true;
            } else if (variant != 0 && variant != 8) return PRISM_ERR_UNSUPPORTED;
        }
        const int64_t kblocks = (K + kDecodeKBlock - 1) / kDecodeKBlock;
        // Packed tiles with more K-slices for the tiles in slow units (s_slow against s): gated, at most 16 rows,
        // nothing forced but perhaps the packed variant itself, N a multiple of 1024 (a tile keeps its unit over
        // all rows, and 16 tiles hold each unit once), every workgroup on a CU of its own.  s as for a plain call
        // with these tiles; s_slow = s + max(1, (2 s + 2) / 5) (the slow stripes need 1.4 times as long).
        StreamPartition balanced{};
        int64_t balanced_slow = 0;
        // Narrow outputs (at most 32 packed tiles): the packed tile with equal slices.  The two-tile form would put
        // half as many workgroups to work, and the balanced form below so many slices that the exchange outweighs what
        // the slow stripes lose (16 x 4096 x 1024: 11.3 us packed in 8 slices, 12.8 us as two tiles, 13.2 us balanced
        // 8 : 11; 16 x 4096 x 2048: 12.9 / 13.9 / 14.6 us; 16 x 2048 x 2048: 10.6 to 11 / 10.6 / 12.4 us).
        const bool narrow = gated && M <= kDecodeMaxRows && N <= 32 * (kDecodeTileN / 2);
        if (narrow && variant == 0 && forced_split <= 0) packed = true;
        if (!narrow && gated && M <= kDecodeMaxRows && (variant == 0 || packed) && forced_split <= 0 && (N * 2) % 2048 == 0 &&
            (g_slow_units.load() & 0xFFFF) != 0) {
            const uint32_t units = (uint32_t)g_slow_units.load() & 0xFFFFu;
            const int64_t nt = N / (kDecodeTileN / 2), n_slow = nt / 16 * __builtin_popcount(units);
            const int64_t cus = cu_count();
            int64_t sb = std::min<int64_t>((cus + nt / 2) / nt, std::min<int64_t>(8, kblocks / 4)), ss = 0;  // the loop below takes it down to what fits
            for (; sb >= 1; --sb) {
                ss = sb + std::max<int64_t>(1, (2 * sb + 2) / 5);
                if (nt * sb + n_slow * (ss - sb) <= cus) break;
            }
            const uint64_t G = (uint64_t)(nt * sb + n_slow * (ss - sb)), T = G * (uint64_t)kblocks;
            const uint64_t run_rows = (uint64_t)((kblocks + std::max<int64_t>(sb, 1) - 1) / std::max<int64_t>(sb, 1)) * kDecodeKBlock + 8;
            // Against the two-tile form: as many workgroups at work as it would have (its grid of 128-column tiles
            // x K-slices, at most one per CU).
            // Measured, packed and balanced against two tiles (us): 8 x 4096 x 14336 40.7 / 42.1, 16 x 1024 x 4096
            // 11.9 / 13.1, 8 x 4096 x 11264 34.4 / 39.8, 8 x 4096 x 7168 24.7 / 29.5; but 8 x 4096 x 4096 (200
            // workgroups against 256) 18.9 / 17.1 and 4 x 8192 x 8192 (144 against 256) 73 / 49.
            const int64_t n128 = (N + kDecodeTileN - 1) / kDecodeTileN;
            int64_t s2 = (cus + n128 / 2) / n128;
            if (n128 * s2 > cus && n128 <= cus) s2 = cus / n128;
            s2 = std::max<int64_t>(1, std::min<int64_t>(s2, std::min<int64_t>(8, kblocks / 8)));
            const int64_t two_tile = std::min<int64_t>(n128 * s2, cus);
            const bool worth = packed || (int64_t)G >= two_tile;
            if (worth && sb >= 1 && nt <= kMaxTickets && ss <= kblocks && ss + 0 <= (int64_t)kStreamMaxSlices && T < (1ull << 31) &&
                (uint64_t)ss * 2 * M * N * 4 < kTwoGiB && run_rows * (uint64_t)N * 2 < kTwoGiB) {
                balanced = StreamPartition{(uint32_t)G, (uint32_t)kblocks, (uint32_t)nt, units, 16u, (uint32_t)sb,
                                           (uint32_t)ss, (uint32_t)kblocks, 0u};
                balanced_slow = ss;
                packed = true;
            }
        }
        const int64_t row_blocks = (M + 16 * row_groups - 1) / (16 * row_groups);
        const int64_t tile_cols = packed ? kDecodeTileN / 2 : kDecodeTileN;
        const int64_t n_tiles = (N + tile_cols - 1) / tile_cols;
        if (row_blocks > 65535 || n_tiles * row_blocks > kMaxTickets) return PRISM_ERR_UNSUPPORTED;
        int64_t S = forced_split;
        if (balanced.G != 0) S = balanced.w_fast;
        if (S <= 0) {
            // About one workgroup per CU (measured best on MI355X: more slices only add partial-sum
            // traffic and tickets), each wavefront keeping at least one K-block.
            const int64_t target = cu_count();
            const int64_t wgs = n_tiles * row_blocks;
            // The multi-row kernel fits one workgroup per CU: never more workgroups than CUs if that can be helped.
            // The 16-row kernel: the nearest number of slices, but never a grid that needs a second round for a few
            // workgroups (X[16,4096] . W[4096,11008], 86 tiles: 20.8 us with 2 slices, 27.7 us with 3; W[4096,7168],
            // 56 tiles: 14.9 us with 4, 20.3 us with 5).
            S = (row_groups > 1) ? target / wgs : (target + wgs / 2) / wgs;
            if (row_groups == 1 && wgs * S > target && wgs <= target) S = target / wgs;
            // 129 to 159 tiles: one slice per tile leaves more than a third of the CUs idle and two make a second
            // round of a few workgroups; three (1.5 to 1.9 rounds of shorter workgroups, dealt out as CUs free up)
            // are faster than both when K is deep enough (W[4096,18432], 144 tiles: 34.9 / 40.2 / 32.0 us with
            // 1 / 2 / 3 slices; W[2048,20352]: 18.0 / 22.4 / 19.6 us).
            if (row_groups == 1 && S == 1 && wgs > target / 2 && wgs < target * 5 / 8 && kblocks >= 96) S = 3;
            // Between one and two rounds of workgroups, the second round should not be a nearly empty one.  If
            // one slice per tile fills less than 77 % of the two rounds, take the 2, 3 or 4 slices that fill theirs
            // best (shorter workgroups, a shorter last round): W[4096,33280], 260 tiles, 68.3 us unsplit, 57.7 us
            // with 4 slices; W[4096,40960], 320 tiles, 72.2 / 65.1 us; W[4096,49152], 384 tiles, 76.0 us, 73.7 us
            // with 2 slices; but W[4096,51200], 400 tiles, 76.3 us unsplit against 81.5 us with 3, and from 512
            // tiles on (520, 640 tiles measured) slices change nothing or cost time.
            // The multi-row kernel, a little over one round (260 tiles: 101.1 -> 99.8 us plain with 64 rows, 161.3 ->
            // 148.3 us gated with 32 rows; 320 tiles are better left unsplit: 93.7 against 95.1 us).
            if (row_groups > 1 && S <= 1 && wgs > target && wgs * 10 < target * 12 && kblocks >= 32) S = 2;
            if (row_groups == 1 && S == 1 && wgs > target && wgs < 2 * target) {
                auto fill = [&](int64_t s) { return (double)(wgs * s) / (double)(target * ((wgs * s + target - 1) / target)); };
                if (fill(1) < 0.77) {
                    int64_t best = 1;
                    for (int64_t s2 = 2; s2 <= 4 && kblocks / s2 >= 16; ++s2)
                        if (fill(s2) > fill(best) + 1e-9) best = s2;
                    S = best;
                }
            }
            int64_t s_max = kblocks / waves;
            if (row_groups == 1) {
                // Measured over shapes from 2 to 235 MB of weights streamed from HBM (an exhaustive run of the
                // tuner): never more than eight slices (the last arrival reads eight slices' partials in one
                // round trip), and a slice keeps at least four K-blocks (eight when gated: two matrices), even
                // if that leaves wavefronts idle.
                s_max = std::min<int64_t>(8, std::max<int64_t>(1, kblocks / ((gated && !packed) ? 8 : 4)));
                // Few column tiles and a deep K (one weight matrix): eight slices leave at least half the CUs idle and
                // every workgroup with a long walk; sixteen, read back in two batches, are faster when a slice still
                // has 16 K-blocks (32 with sixteen tiles): 16 x 8192 x 512 11.3 -> 8.7 us, 16 x 16384 x 1024 18.5 ->
                // 13.3 us, 16 x 16384 x 2048 20.2 -> 17.8 us; but 16 x 4096 x 1024 8.3 -> 9.0 us, 16 x 8192 x 2048 12.4
                // -> 12.8 us.
                if (!gated && n_tiles * 8 <= target / 2 && kblocks >= 16 * (n_tiles <= 8 ? 16 : 32)) s_max = 16;
            }
            if (S > s_max) S = s_max;
            if (S < 1) S = 1;
        }
        if (S > kblocks) S = kblocks;
        // Unsplit plain calls run a little faster with four wavefronts per workgroup (half the LDS reduction, two
        // workgroups can share a CU): 0.5 to 3 % on eight shapes from W[2048,32768] to W[8192,57344].
        if (row_groups == 1 && M <= kDecodeMaxRows && variant == 0 && !gated && S == 1 && forced_split <= 0) waves = 4;
        // Byte offsets inside one K-slice must fit in 31 bits: a weight matrix of 2 GiB or more is cut
        // into more slices (unless the split was forced).
        auto slice_fits = [&](int64_t s) {
            const uint64_t slice_rows = (uint64_t)((kblocks + s - 1) / s) * kDecodeKBlock + 8;
            return slice_rows * (uint64_t)N * 2 < kTwoGiB;
        };
        if (forced_split <= 0)
            while (!slice_fits(S) && S < kblocks) S = std::min<int64_t>(kblocks, 2 * S);
        if (S > 65535 || !slice_fits(S)) return PRISM_ERR_UNSUPPORTED;
        // The partial sums are addressed with 31-bit byte offsets.
        auto partials_fit = [&](int64_t s) { return (uint64_t)s * (gated ? 2 : 1) * M * N * 4 < kTwoGiB; };
        if (forced_split <= 0)
            while (S > 1 && !partials_fit(S)) --S;
        if (S > 1 && !partials_fit(S)) return PRISM_ERR_UNSUPPORTED;
        if (!slice_fits(S)) return PRISM_ERR_UNSUPPORTED;
        // The two-pass weighted partition (an option, mode bit 0): for 129 to 159 column tiles, 256 workgroups with
        // equal shares of all K-blocks, a share of at least four K-blocks (eight when gated).  A workgroup whose
        // share spans two tiles makes two passes and pays the reduction twice, which is why it is not the default:
        // W[4096,18432] 35.2 us against 32.0 us with three slices per tile, X[16,4096] . W[4096,11008] 24.8 us against
        // 20.8 us as 86 x 2.  In the partition, 256-byte tiles that contain a slow unit weigh 5 : 4 if mode bit 1 is
        // set and the row pitch keeps a tile in its units.
        StreamPartition sp{};
        int64_t s_pitch = S;
        if (balanced.G != 0) {
            sp = balanced;
            s_pitch = balanced_slow;
        } else if (row_groups == 1 && forced_split <= 0 && (g_stream_mode.load() & 1) != 0 && n_tiles > cu_count() / 2 &&
                   n_tiles < cu_count() * 5 / 8) {
            // slot j (256 bytes) holds units 2j and 2j + 1
            uint32_t slow = 0;
            if (!packed && (g_stream_mode.load() & 2) != 0 && (N * 2) % 2048 == 0 && n_tiles % 8 == 0)
                for (int j = 0; j < 8; ++j)
                    if ((g_slow_units.load() >> (2 * j)) & 3) slow |= 1u << j;
            StreamPartition cand{0u, (uint32_t)kblocks, (uint32_t)n_tiles, slow, 8u, 4u, 5u, 0u, 0u};
            const uint64_t T = sp_total(cand);
            int64_t G = std::min<int64_t>(cu_count(), std::min<int64_t>(n_tiles * kblocks / ((gated && !packed) ? 8 : 4), 8 * n_tiles));
            if (G < 1) G = 1;
            if (T < (1ull << 31) && n_tiles < (1 << 24)) {
                const uint64_t q = T / G;
                // A tile's weight units meet at most this many workgroups' ranges.
                int64_t most = (int64_t)(((slow ? 5u : 4u) * (uint64_t)kblocks + q - 1) / q) + 1;
                if (!slow && T % G == 0 && (q % (4 * kblocks) == 0 || (4 * kblocks) % q == 0))
                    most = std::max<int64_t>(1, 4 * kblocks / q);  // the ranges line up with the tiles
                // Byte offsets inside one run of K-blocks must fit in 31 bits, as for a K-slice.
                const uint64_t run_rows = std::min<uint64_t>(kblocks, q / 4 + 2) * kDecodeKBlock + 8;
                // q < a tile's weight: a workgroup's range (q or q + 1 units) meets at most two tiles.
                if (q < 4 * (uint64_t)kblocks && most <= kStreamMaxSlices && partials_fit(most) &&
                    run_rows * (uint64_t)N * 2 < kTwoGiB) {
                    sp = cand;
                    sp.G = (uint32_t)G;
                    sp.q = (uint32_t)q;
                    sp.r = (uint32_t)(T % G);
                    s_pitch = most;
                }
            }
        }
        // Measured (us, X through LDS against straight loads): 512 x 4096 x 4096 32.1 / 34.1, 256 x 14336 x 4096
        // 56.6 / 65.5, 1024 x 4096 x 6144 85.4 / 92.7; with slices of 16 K-blocks (64 x 4096 x 4096) 18.3 / 16.7.
        // A single row block whose row groups are less than three quarters full moves padding through LDS for nothing
        // (17 rows in a 32-row workgroup: 2 to 7 % slower on five shapes; 24 of 32 and 48 of 64: even).
        if (row_groups > 1 && !gated && variant == 0 && kblocks / std::max<int64_t>(1, S) >= 64 &&
            (row_blocks > 1 || M * 4 >= 3 * 16 * row_groups))
            xlds = true;
        out->waves = waves;
        out->row_groups = row_groups;
        out->xlds = xlds;
        out->packed = packed;
        out->sp = sp;
        out->base_split = (int)S;
        p.split_k = (int32_t)S;
        p.tile_m = 16 * row_groups;
        p.tile_n = (int32_t)tile_cols;
        p.grid_x = (int32_t)n_tiles;
        p.grid_y = (int32_t)S;
        if (sp.G != 0) {
            S = s_pitch;  // the most workgroups that share a tile: the slices the workspace holds
            p.split_k = (int32_t)S;
            p.grid_x = (int32_t)sp.G;
            p.grid_y = 1;
        }
        p.grid_z = (int32_t)row_blocks;
        p.block = waves * 64;
        if (S > 1) {
            out->ss_bytes = round_up((uint64_t)n_tiles * row_blocks * S * 16 * row_groups * 4, 256);
            p.workspace_bytes = PRISM_WORKSPACE_HEADER_BYTES + out->ss_bytes +
                                (uint64_t)S * (gated ? 2 : 1) * M * N * 4;
        }
        return PRISM_OK;
    }

    // PRISM_PATH_PREFILL
    if ((uint64_t)K * N * 2 >= kTwoGiB) return PRISM_ERR_UNSUPPORTED;
    int bm = 0, bn = 0;
    choose_prefill_tile(gated, M, N, variant, &bm, &bn);
    if (!prefill_tile_known(gated, bm, bn)) return PRISM_ERR_UNSUPPORTED;
    const int cw = gated ? bn / 2 : bn;
    const int64_t tiles = ((M + bm - 1) / bm) * ((N + cw - 1) / cw);
    if (tiles > 0x7FFFFFFF) return PRISM_ERR_UNSUPPORTED;
    p.tile_m = bm;
    p.tile_n = bn;
    p.grid_x = (int32_t)tiles;
    p.grid_y = 1;
    p.block = 256;
    return PRISM_OK;
}

prism_status_t make_plan(prism_op_t op, int64_t M, int64_t K, int64_t N, prism_dtype_t dtype, Plan* out) {
    if (op != PRISM_OP_RMSNORM_MATMUL && op != PRISM_OP_RMSNORM_GATED_MLP && op != PRISM_OP_SOFTMAX_MATMUL)
        return PRISM_ERR_UNSUPPORTED;
    return make_plan_with(op, M, K, N, dtype, resolve_choice(op, M, K, N, dtype), out);
}

// Attention: the matrix-core kernel for 16-bit storage, head dimension 128 and at most 16 query heads per
// batch entry; the plain kernel otherwise (head dimension up to 1024).
prism_status_t make_attention_plan(int64_t B, int64_t G, int64_t H, int64_t D, prism_dtype_t dtype, AttentionPlan* p) {
    if (!dtype_known(dtype)) return PRISM_ERR_UNSUPPORTED;
    if (B < 0 || G < 0 || H <= 0 || D <= 0) return PRISM_ERR_INVALID_ARG;
    *p = AttentionPlan{PRISM_PATH_SIMPLE, 1, 0, 0};
    if (B == 0 || G == 0) return PRISM_OK;
    if (B > 65535 || G > 65535 || D > 1024 || H > 0x7FFFFFFF / 2048) return PRISM_ERR_UNSUPPORTED;
    const int forced = g_override.path.load();
    if (forced != PRISM_PATH_AUTO && forced != PRISM_PATH_SIMPLE && forced != PRISM_PATH_ATTENTION) return PRISM_ERR_UNSUPPORTED;
    const bool fast_ok = dtype != PRISM_F32 && D == kAttnHeadDim && G <= kAttnMaxHeads;
    if (forced == PRISM_PATH_ATTENTION && !fast_ok) return PRISM_ERR_UNSUPPORTED;
    if (forced == PRISM_PATH_SIMPLE || !fast_ok) return PRISM_OK;
    p->path = PRISM_PATH_ATTENTION;
    int64_t keys = kAttnSliceKeys;
    const int forced_split = g_override.split_k.load();
    int64_t S = forced_split;
    if (S <= 0) {
        // 128 keys per workgroup (one 32-key block per wavefront) up to eight slices, which the combining
        // workgroup reads in one round trip; longer contexts get longer slices first and more of them later
        // (measured with two batch entries of eight heads: 1024 keys 8.1 us in 8 slices, 8.7 in 16; 2048 keys
        // 9.3 us in 16, 10.0 in 8; 4096 keys 11.5 us in 16, 12.0 in 32; 8192 keys 14.2 us in 32, 14.9 in 16;
        // 32768 keys 22.3 us in 64, 23.7 in 32; 131072 keys 46 us in 64, 65 in 32).
        S = (H + keys - 1) / keys;
        if (S > 8) S = H <= 1536 ? 8 : (H <= 6144 ? 16 : (H <= 16384 ? 32 : 64));
        // Never more workgroups than CUs over all batch entries: with 32 batch entries and 16 heads, 2048 keys take
        // 13.9 us in 8 slices and 19.4 us in 16; 16384 keys 45.8 us in 8 and 67.7 us in 32.
        // With more batch entries than CUs the workgroups come in rounds anyway, and long contexts still gain from
        // four slices (300 entries, 4096 keys: 137.6 us unsplit, 110.7 us in 4 slices).
        // (128 entries fill the CUs with two slices each: 4096 keys 43.6 us in 2, 46.8 us in 4; 16384 keys 152.6 / 161.1 us)
        const int64_t per_entry = cu_count() / B;
        S = std::min<int64_t>(S, per_entry >= 2 ? per_entry : (H >= 4096 ? 4 : (H >= 2048 ? 2 : 1)));
    }
    if (S > kAttnMaxSlices) S = kAttnMaxSlices;
    keys = ((H + S - 1) / S + 31) / 32 * 32;
    S = (H + keys - 1) / keys;  // no empty slice
    if (S > 1 && (uint64_t)B * S * 16 * kAttnHeadDim * 4 >= kTwoGiB) {
        // 31-bit offsets into the partials: a batch this large is left to the plain kernel
        if (forced == PRISM_PATH_ATTENTION) return PRISM_ERR_UNSUPPORTED;
        *p = AttentionPlan{PRISM_PATH_SIMPLE, 1, 0, 0};
        return PRISM_OK;
    }
    p->splits = (int)S;
    p->slice_keys = (int)keys;
    if (S > 1) p->workspace_bytes = PRISM_WORKSPACE_HEADER_BYTES + (uint64_t)B * S * 16 * (2 + kAttnHeadDim) * 4;
    return PRISM_OK;
}

bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

// A plain grid of 128-column tiles over a W whose row pitch is a multiple of 2 KiB: every tile keeps its two 128-byte
// address units over all rows, and the tiles in slow units (prism_set_stream_balance) take about 1.4 times as long.
// When the grid needs more than one round of workgroups, those tiles are started first (decode_kernel.hip); which
// residues of the tile number modulo 8 they are depends on where W starts.
StreamPartition slow_tiles_first(const void* W, const void* W2, int64_t N, int64_t n_tiles, int64_t split, bool packed) {
    StreamPartition sp{};
    const uint32_t units = (uint32_t)g_slow_units.load() & 0xFFFFu;
    if (units == 0 || packed || (N * 2) % 2048 != 0 || n_tiles % 8 != 0 || ((uintptr_t)W & 255u) != 0 || n_tiles * split <= cu_count() ||
        (W2 && (((uintptr_t)W ^ (uintptr_t)W2) & 2047u) != 0))
        return sp;
    const uint32_t first_pair = (uint32_t)(((uintptr_t)W >> 8) & 7u);  // tile t covers units 2 (first_pair + t) mod 16, + 1
    uint32_t mask = 0;
    for (uint32_t r = 0; r < 8; ++r)
        if ((units >> (2u * ((first_pair + r) & 7u))) & 3u) mask |= 1u << r;
    if (mask == 0 || mask == 0xFFu) return sp;
    sp.slow = mask;
    sp.period = 8;
    return sp;
}

// One call of the family: `flags` says which optional steps it takes (gain is dropped here when g
// is null).
prism_status_t run(prism_op_t op, const void* X, const void* g, const void* W1, const void* W2, void* Y, int64_t M,
                   int64_t K, int64_t N, float eps, prism_dtype_t dtype, hipStream_t stream,
                   int flags = kFlagGain | kFlagNorm | kFlagSilu, bool use_static_scratch = false) {
    const bool gated = op == PRISM_OP_RMSNORM_GATED_MLP;
    if (!g) flags &= ~kFlagGain;
    if (!dtype_known(dtype)) return PRISM_ERR_UNSUPPORTED;
    if (M < 0 || N < 0 || K <= 0) return PRISM_ERR_INVALID_ARG;
    if (!(eps >= 0.0f) || !std::isfinite(eps)) return PRISM_ERR_INVALID_ARG;
    if (M == 0 || N == 0) return PRISM_OK;  // empty problem: pointers are not looked at
    if (!X || !W1 || !Y || (gated && !W2)) return PRISM_ERR_INVALID_ARG;
    if (!aligned16(X) || !aligned16(g) || !aligned16(W1) || !aligned16(Y) || (gated && !aligned16(W2)))
        return PRISM_ERR_INVALID_ARG;
    Plan plan;
    const prism_status_t st = make_plan(op, M, K, N, dtype, &plan);
    if (st != PRISM_OK) return st;

    Call c{X, g, W1, gated ? W2 : nullptr, Y, (int)M, (int)K, (int)N, eps, gated, flags, stream};
    hipError_t err = hipSuccess;
    switch (plan.pub.path) {
        case PRISM_PATH_SIMPLE:
            err = (dtype == PRISM_F32) ? launch_simple_f32(c)
                  : (dtype == PRISM_F16) ? launch_simple_f16(c) : launch_simple_bf16(c);
            break;
        case PRISM_PATH_DECODE: {
            DecodeWorkspace ws{nullptr, nullptr, nullptr};
            if (plan.pub.split_k > 1) {
                Workspace w{nullptr, 0};
                if (use_static_scratch) {
                    if (plan.pub.workspace_bytes > PRISM_STATIC_SCRATCH_BYTES) return PRISM_ERR_WORKSPACE;
                    if (const prism_status_t s = static_scratch(stream, &w); s != PRISM_OK) return s;
                } else if (const prism_status_t s = workspace_for(stream, &w); s != PRISM_OK) {
                    return s;
                }
                if (!w.ptr || w.bytes < plan.pub.workspace_bytes) return PRISM_ERR_WORKSPACE;
                char* base = (char*)w.ptr;
                ws.tickets = (unsigned*)base;
                ws.ss_part = (float*)(base + PRISM_WORKSPACE_HEADER_BYTES);
                ws.acc_part = (float*)(base + PRISM_WORKSPACE_HEADER_BYTES + plan.ss_bytes);
            }
            // The units are read off the address of W: tile j's unit is that of tile 0 plus j (128-byte tiles) or
            // its pair of units (256-byte tiles).  W off a tile boundary, or W2 out of step with W1, gets equal
            // shares: the plain grid for the packed tile, equal weights in the partition.
            StreamPartition sp = plan.sp;
            int split = plan.pub.split_k;
            if (sp.G != 0 && sp.slow != 0) {
                const uintptr_t a1 = reinterpret_cast<uintptr_t>(W1), a2 = reinterpret_cast<uintptr_t>(W2);
                const uintptr_t tile_bytes = plan.packed ? 128u : 256u;
                const bool aligned = (a1 & (tile_bytes - 1)) == 0 && (!gated || ((a1 ^ a2) & 2047u) == 0);
                if (aligned) {
                    const unsigned first = (unsigned)(a1 / tile_bytes) & (sp.period - 1u), mask = (1u << sp.period) - 1u;
                    sp.slow = ((sp.slow >> first) | (sp.slow << (sp.period - first))) & mask;
                } else if (plan.packed) {
                    sp = StreamPartition{};
                    split = plan.base_split;
                } else {
                    sp.slow = 0;
                    const uint64_t T = sp_total(sp);
                    sp.q = (uint32_t)(T / sp.G);
                    sp.r = (uint32_t)(T % sp.G);
                }
            }
            if (plan.row_groups == 1 && sp.G == 0) sp = slow_tiles_first(W1, gated ? W2 : nullptr, N, plan.pub.grid_x, split, plan.packed);
            err = plan.row_groups > 1
                      ? launch_decode_rows_16bit(c, dtype == PRISM_F16, plan.pub.split_k, plan.row_groups, plan.xlds, ws)
                      : launch_decode_16bit(c, dtype == PRISM_F16, split, sp, plan.waves, plan.packed, ws);
            break;
        }
        case PRISM_PATH_PREFILL:
            err = launch_prefill_16bit(c, dtype == PRISM_F16, plan.pub.tile_m, plan.pub.tile_n);
            break;
        default:
            return PRISM_ERR_UNSUPPORTED;
    }
    return err == hipSuccess ? PRISM_OK : PRISM_ERR_HIP;
}

}  // namespace
}  // namespace prism

using namespace prism;

extern "C" {

prism_status_t prism_rmsnorm_matmul(const void* X, const void* g, const void* W, void* Y, int64_t M, int64_t K,
                                    int64_t N, float eps, prism_dtype_t dtype, hipStream_t stream) {
    return run(PRISM_OP_RMSNORM_MATMUL, X, g, W, nullptr, Y, M, K, N, eps, dtype, stream);
}

prism_status_t prism_rmsnorm_matmul_static(const void* X, const void* g, const void* W, void* Y, int64_t M, int64_t K,
                                           int64_t N, float eps, prism_dtype_t dtype, hipStream_t stream) {
    return run(PRISM_OP_RMSNORM_MATMUL, X, g, W, nullptr, Y, M, K, N, eps, dtype, stream,
               kFlagGain | kFlagNorm | kFlagSilu, /*use_static_scratch=*/true);
}

prism_status_t prism_rmsnorm_gated_mlp(const void* X, const void* g, const void* W1, const void* W2, void* Y,
                                       int64_t M, int64_t K, int64_t N, float eps, prism_dtype_t dtype,
                                       hipStream_t stream) {
    return run(PRISM_OP_RMSNORM_GATED_MLP, X, g, W1, W2, Y, M, K, N, eps, dtype, stream);
}

prism_status_t prism_rmsnorm_glu(const void* X, const void* g, const void* W1, const void* W2, void* Y, int64_t M,
                                 int64_t K, int64_t N, float eps, prism_dtype_t dtype, hipStream_t stream) {
    return run(PRISM_OP_RMSNORM_GATED_MLP, X, g, W1, W2, Y, M, K, N, eps, dtype, stream, kFlagGain | kFlagNorm);
}

prism_status_t prism_swiglu(const void* X, const void* W_gate, const void* W_up, void* Y, int64_t M, int64_t K,
                            int64_t N, prism_dtype_t dtype, hipStream_t stream) {
    return run(PRISM_OP_RMSNORM_GATED_MLP, X, nullptr, W_gate, W_up, Y, M, K, N, 0.0f, dtype, stream, kFlagSilu);
}

prism_status_t prism_softmax_matmul(const void* X, const void* W, void* Y, int64_t M, int64_t K, int64_t N,
                                    prism_dtype_t dtype, hipStream_t stream) {
    if (!dtype_known(dtype)) return PRISM_ERR_UNSUPPORTED;
    if (M < 0 || N < 0 || K <= 0) return PRISM_ERR_INVALID_ARG;
    if (M == 0 || N == 0) return PRISM_OK;
    if (!X || !W || !Y) return PRISM_ERR_INVALID_ARG;
    if (!aligned16(X) || !aligned16(W) || !aligned16(Y)) return PRISM_ERR_INVALID_ARG;
    Plan plan;
    const prism_status_t st = make_plan(PRISM_OP_SOFTMAX_MATMUL, M, K, N, dtype, &plan);
    if (st != PRISM_OK) return st;
    const SoftmaxCall c{X, W, Y, (int)M, (int)K, (int)N, stream};
    hipError_t err;
    if (plan.pub.path != PRISM_PATH_ROWS) {
        err = launch_softmax_simple(c, (int)dtype);
    } else if (plan.pub.tile_m == kSoftmaxRows) {
        err = launch_softmax_rows_16bit(c, dtype == PRISM_F16);
    } else {
        SoftmaxWorkspace ws{nullptr, nullptr, nullptr};
        if (plan.pub.split_k > 1) {
            Workspace w{nullptr, 0};
            if (const prism_status_t s = workspace_for(stream, &w); s != PRISM_OK) return s;
            if (!w.ptr || w.bytes < plan.pub.workspace_bytes) return PRISM_ERR_WORKSPACE;
            char* base = (char*)w.ptr;
            ws.tickets = (unsigned*)base;
            ws.ml_part = (float*)(base + PRISM_WORKSPACE_HEADER_BYTES);
            ws.acc_part = (float*)(base + PRISM_WORKSPACE_HEADER_BYTES + plan.ss_bytes);
        }
        err = launch_softmax_split_16bit(c, dtype == PRISM_F16, plan.pub.split_k, ws);
    }
    return err == hipSuccess ? PRISM_OK : PRISM_ERR_HIP;
}

prism_status_t prism_gqa_decode_attention(const void* Q, const void* K, const void* V, void* O, int64_t B, int64_t G,
                                          int64_t H, int64_t D, float scale, int32_t qk_norm, float eps,
                                          prism_dtype_t dtype, hipStream_t stream) {
    if (!std::isfinite(scale) || !(eps >= 0.0f) || !std::isfinite(eps)) return PRISM_ERR_INVALID_ARG;
    AttentionPlan plan;
    const prism_status_t st = make_attention_plan(B, G, H, D, dtype, &plan);
    if (st != PRISM_OK) return st;
    if (B == 0 || G == 0) return PRISM_OK;
    if (!Q || !K || !V || !O) return PRISM_ERR_INVALID_ARG;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O)) return PRISM_ERR_INVALID_ARG;
    const AttentionCall c{Q, K, V, O, (int)B, (int)G, (int)H, (int)D, scale, qk_norm != 0, eps, stream};
    hipError_t err;
    if (plan.path == PRISM_PATH_ATTENTION) {
        AttentionWorkspace ws{nullptr, nullptr, nullptr, nullptr};
        if (plan.splits > 1) {
            Workspace w{nullptr, 0};
            if (const prism_status_t s = workspace_for(stream, &w); s != PRISM_OK) return s;
            if (!w.ptr || w.bytes < plan.workspace_bytes) return PRISM_ERR_WORKSPACE;
            char* base = (char*)w.ptr;
            const uint64_t rows = (uint64_t)B * plan.splits * 16;
            ws.tickets = (unsigned*)base;
            ws.m_part = (float*)(base + PRISM_WORKSPACE_HEADER_BYTES);
            ws.l_part = ws.m_part + rows;
            ws.acc_part = ws.l_part + rows;
        }
        err = launch_gqa_16bit(c, dtype == PRISM_F16, plan, ws);
    } else {
        err = launch_gqa_simple(c, (int)dtype);
    }
    return err == hipSuccess ? PRISM_OK : PRISM_ERR_HIP;
}

uint64_t prism_attention_workspace_bytes(int64_t B, int64_t G, int64_t H, int64_t D, prism_dtype_t dtype) {
    AttentionPlan plan;
    if (make_attention_plan(B, G, H, D, dtype, &plan) != PRISM_OK) return 0;
    return plan.workspace_bytes;
}

prism_status_t prism_attention_plan(int64_t B, int64_t G, int64_t H, int64_t D, prism_dtype_t dtype, prism_plan_t* out) {
    if (!out) return PRISM_ERR_INVALID_ARG;
    AttentionPlan plan;
    const prism_status_t st = make_attention_plan(B, G, H, D, dtype, &plan);
    if (st != PRISM_OK) return st;
    std::memset(out, 0, sizeof(*out));
    out->path = plan.path;
    out->split_k = plan.splits;
    out->tile_m = plan.path == PRISM_PATH_ATTENTION ? 16 : 1;
    out->tile_n = plan.slice_keys;
    out->grid_x = plan.path == PRISM_PATH_ATTENTION ? plan.splits : (int32_t)G;
    out->grid_y = (int32_t)B;
    out->block = 256;
    out->workspace_bytes = plan.workspace_bytes;
    return PRISM_OK;
}

prism_status_t prism_rmsnorm_matmul_bf16(const void* X, const void* g, const void* W, void* Y, int64_t M, int64_t K,
                                         int64_t N, float eps, hipStream_t stream) {
    return run(PRISM_OP_RMSNORM_MATMUL, X, g, W, nullptr, Y, M, K, N, eps, PRISM_BF16, stream);
}

prism_status_t prism_rmsnorm_matmul_f32(const void* X, const void* g, const void* W, void* Y, int64_t M, int64_t K,
                                        int64_t N, float eps, hipStream_t stream) {
    return run(PRISM_OP_RMSNORM_MATMUL, X, g, W, nullptr, Y, M, K, N, eps, PRISM_F32, stream);
}

prism_status_t prism_rmsnorm_gated_mlp_bf16(const void* X, const void* g, const void* W1, const void* W2, void* Y,
                                            int64_t M, int64_t K, int64_t N, float eps, hipStream_t stream) {
    return run(PRISM_OP_RMSNORM_GATED_MLP, X, g, W1, W2, Y, M, K, N, eps, PRISM_BF16, stream);
}

prism_status_t prism_rmsnorm_gated_mlp_f32(const void* X, const void* g, const void* W1, const void* W2, void* Y,
                                           int64_t M, int64_t K, int64_t N, float eps, hipStream_t stream) {
    return run(PRISM_OP_RMSNORM_GATED_MLP, X, g, W1, W2, Y, M, K, N, eps, PRISM_F32, stream);
}

uint64_t prism_workspace_bytes(prism_op_t op, int64_t M, int64_t K, int64_t N, prism_dtype_t dtype) {
    Plan plan;
    if (make_plan(op, M, K, N, dtype, &plan) != PRISM_OK) return 0;
    return plan.pub.workspace_bytes;
}

prism_status_t prism_set_workspace(void* dev_ptr, uint64_t bytes) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return PRISM_ERR_HIP;
    if (dev < 0 || dev >= kMaxDevices) return PRISM_ERR_UNSUPPORTED;
    if (!dev_ptr || bytes == 0) {
        std::lock_guard<std::mutex> lock(g_ws_mutex);
        g_workspace[dev] = Workspace{nullptr, 0};
        return PRISM_OK;
    }
    if (((uintptr_t)dev_ptr & 255u) != 0 || bytes < PRISM_WORKSPACE_HEADER_BYTES) return PRISM_ERR_INVALID_ARG;
    if (hipMemset(dev_ptr, 0, PRISM_WORKSPACE_HEADER_BYTES) != hipSuccess) return PRISM_ERR_HIP;
    if (hipDeviceSynchronize() != hipSuccess) return PRISM_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_ws_mutex);
    g_workspace[dev] = Workspace{dev_ptr, bytes};
    return PRISM_OK;
}

prism_status_t prism_set_stream_workspace(hipStream_t stream, void* dev_ptr, uint64_t bytes) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return PRISM_ERR_HIP;
    if (dev < 0 || dev >= kMaxDevices) return PRISM_ERR_UNSUPPORTED;
    const bool unregister = !dev_ptr || bytes == 0;
    if (!unregister) {
        if (((uintptr_t)dev_ptr & 255u) != 0 || bytes < PRISM_WORKSPACE_HEADER_BYTES) return PRISM_ERR_INVALID_ARG;
        if (hipMemset(dev_ptr, 0, PRISM_WORKSPACE_HEADER_BYTES) != hipSuccess) return PRISM_ERR_HIP;
        if (hipDeviceSynchronize() != hipSuccess) return PRISM_ERR_HIP;
    }
    std::lock_guard<std::mutex> lock(g_ws_mutex);
    int slot = -1;
    for (int i = 0; i < g_stream_ws_count; ++i)
        if (g_stream_ws[i].dev == dev && g_stream_ws[i].stream == stream) slot = i;
    if (unregister) {
        if (slot >= 0) g_stream_ws[slot] = g_stream_ws[--g_stream_ws_count];
        return PRISM_OK;
    }
    if (slot < 0) {
        if (g_stream_ws_count == kMaxStreamWorkspaces) return PRISM_ERR_UNSUPPORTED;
        slot = g_stream_ws_count++;
    }
    g_stream_ws[slot] = StreamWorkspace{dev, stream, Workspace{dev_ptr, bytes}};
    return PRISM_OK;
}

prism_status_t prism_plan(prism_op_t op, int64_t M, int64_t K, int64_t N, prism_dtype_t dtype, prism_plan_t* plan) {
    if (!plan) return PRISM_ERR_INVALID_ARG;
    Plan p;
    const prism_status_t st = make_plan(op, M, K, N, dtype, &p);
    if (st == PRISM_OK) *plan = p.pub;
    return st;
}

prism_status_t prism_set_override(int32_t path, int32_t split_k, int32_t variant) {
    if (path < PRISM_PATH_AUTO || path > PRISM_PATH_ATTENTION || split_k < 0 || variant < 0) return PRISM_ERR_INVALID_ARG;
    g_override.path.store(path);
    g_override.split_k.store(split_k);
    g_override.variant.store(variant);
    return PRISM_OK;
}

prism_status_t prism_plan_table_set(prism_op_t op, int64_t M, int64_t K, int64_t N, prism_dtype_t dtype, int32_t path,
                                    int32_t split_k, int32_t variant) {
    if (path < PRISM_PATH_AUTO || path > PRISM_PATH_ROWS || split_k < 0 || variant < 0) return PRISM_ERR_INVALID_ARG;
    if (M <= 0 || N <= 0) return PRISM_ERR_INVALID_ARG;
    // An assignment that cannot run this shape is refused here, not at the call.
    Plan probe;
    const prism_status_t st = make_plan_with(op, M, K, N, dtype, Choice{path, split_k, variant}, &probe);
    if (st != PRISM_OK) return st;
    std::lock_guard<std::mutex> lock(g_table_mutex);
    int slot = g_table_size;
    for (int i = 0; i < g_table_size; ++i) {
        const TableEntry& e = g_table[i];
        if (e.op == (int32_t)op && e.dtype == (int32_t)dtype && e.M == M && e.K == K && e.N == N) slot = i;
    }
    if (slot == kTableCapacity) return PRISM_ERR_UNSUPPORTED;
    g_table[slot] = TableEntry{(int32_t)op, (int32_t)dtype, M, K, N, Choice{path, split_k, variant}};
    if (slot == g_table_size) ++g_table_size;
    return PRISM_OK;
}

prism_status_t prism_plan_table_clear(void) {
    std::lock_guard<std::mutex> lock(g_table_mutex);
    g_table_size = 0;
    return PRISM_OK;
}

int32_t prism_plan_table_size(void) {
    std::lock_guard<std::mutex> lock(g_table_mutex);
    return g_table_size;
}

prism_status_t prism_set_stream_balance(int32_t slow_units, int32_t mode) {
    if (slow_units < 0 || slow_units > 0xFFFF || mode < 0 || mode > 3) return PRISM_ERR_INVALID_ARG;
    g_slow_units.store(slow_units);
    g_stream_mode.store(mode);
    return PRISM_OK;
}

prism_status_t prism_stream_partition_blocks(int32_t workgroups, int32_t kblocks, int32_t n_tiles, int32_t slow_tiles,
                                            int32_t period, int32_t w_fast, int32_t w_slow, int32_t wg, int32_t tile,
                                            int32_t* first, int32_t* count) {
    if (!first || !count || workgroups < 1 || workgroups > 65535 || kblocks < 1 || n_tiles < 1 ||
        (period != 8 && period != 16) || slow_tiles < 0 || slow_tiles >= (1 << period) || w_fast < 1 || w_slow < w_fast ||
        w_slow > 64 || wg < 0 || wg >= workgroups || tile < 0 || tile >= n_tiles)
        return PRISM_ERR_INVALID_ARG;
    StreamPartition sp{(uint32_t)workgroups, (uint32_t)kblocks, (uint32_t)n_tiles, (uint32_t)slow_tiles, (uint32_t)period,
                       (uint32_t)w_fast, (uint32_t)w_slow, 0u, 0u};
    const uint64_t T = sp_total(sp);
    if (T >= (1ull << 31)) return PRISM_ERR_UNSUPPORTED;
    sp.q = (uint32_t)(T / sp.G);
    sp.r = (uint32_t)(T % sp.G);
    uint32_t r0 = 0, r1 = 0;
    sp_blocks(sp, (uint32_t)wg, (uint32_t)tile, r0, r1);
    *first = (int32_t)r0;
    *count = r1 > r0 ? (int32_t)(r1 - r0) : 0;
    return PRISM_OK;
}

prism_status_t prism_probe_stream(const void* W, const void* W2, int64_t K, int64_t N, int32_t split_k,
                                  hipStream_t stream) {
    if (K <= 0 || N <= 0 || split_k < 1) return PRISM_ERR_INVALID_ARG;
    if (!W || !aligned16(W) || !aligned16(W2)) return PRISM_ERR_INVALID_ARG;
    const int64_t kblocks = (K + kDecodeKBlock - 1) / kDecodeKBlock;
    const int64_t n_tiles = (N + kDecodeTileN - 1) / kDecodeTileN;
    if (N % 8 != 0 || split_k > kblocks || split_k > 65535 || n_tiles > 0x7FFFFFFF) return PRISM_ERR_UNSUPPORTED;
    // byte offsets inside a slice fit in 31 bits, as for the decode kernel
    if ((uint64_t)((kblocks + split_k - 1) / split_k * kDecodeKBlock + 8) * (uint64_t)N * 2 >= kTwoGiB) return PRISM_ERR_UNSUPPORTED;
    Workspace w{nullptr, 0};
    if (const prism_status_t s = workspace_for(stream, &w); s != PRISM_OK) return s;
    if (!w.ptr || w.bytes < 2ull * PRISM_WORKSPACE_HEADER_BYTES) return PRISM_ERR_WORKSPACE;
    // the probe's one possible store goes past the arrival counters
    unsigned* sink = (unsigned*)((char*)w.ptr + PRISM_WORKSPACE_HEADER_BYTES);
    return launch_probe_stream(W, W2, sink, (int)K, (int)N, split_k, stream) == hipSuccess ? PRISM_OK : PRISM_ERR_HIP;
}

prism_status_t prism_probe_units(const void* base, uint64_t bytes, int32_t groups, uint64_t* ticks, hipStream_t stream) {
    if (!base || !ticks || ((uintptr_t)base & 2047u) != 0 || ((uintptr_t)ticks & 7u) != 0 || groups < 1 || groups > 4096)
        return PRISM_ERR_INVALID_ARG;
    const uint64_t blocks_per_group = bytes / 2048 / (uint64_t)groups;
    if (blocks_per_group < 1) return PRISM_ERR_INVALID_ARG;
    if (blocks_per_group >= (1u << 20)) return PRISM_ERR_UNSUPPORTED;  // 31-bit offsets inside a group
    return launch_probe_units(base, (unsigned)blocks_per_group, groups, (unsigned long long*)ticks, stream) == hipSuccess
               ? PRISM_OK : PRISM_ERR_HIP;
}

prism_status_t prism_probe_loads(const void* base, uint64_t bytes, int32_t pattern, int32_t reps, int32_t workgroups,
                                 uint64_t* ticks, hipStream_t stream) {
    if (!base || !ticks || !aligned16(base) || ((uintptr_t)ticks & 7u) != 0 || pattern < 0 || pattern > 3 || reps < 1 ||
        reps > 4096 || workgroups < 1 || workgroups > 65535 || bytes < PRISM_PROBE_LOADS_BYTES)
        return PRISM_ERR_INVALID_ARG;
    return launch_probe_loads(base, pattern, reps, workgroups, (unsigned long long*)ticks, stream) == hipSuccess
               ? PRISM_OK : PRISM_ERR_HIP;
}

prism_status_t prism_probe_linear(const void* base, uint64_t bytes, int32_t workgroups, void* sink, hipStream_t stream) {
    if (!base || !sink || !aligned16(base) || workgroups < 1 || workgroups > 65535 || bytes < 1024ull * (uint64_t)workgroups ||
        bytes % 16 != 0)
        return PRISM_ERR_INVALID_ARG;
    if (bytes / (uint64_t)workgroups + 1024 >= kTwoGiB) return PRISM_ERR_UNSUPPORTED;  // 31-bit offsets inside a piece
    return launch_probe_linear(base, bytes, workgroups, (unsigned*)sink, stream) == hipSuccess ? PRISM_OK : PRISM_ERR_HIP;
}

prism_status_t prism_probe_mfma(void* sink, int32_t workgroups, int32_t iters, hipStream_t stream) {
    if (!sink || workgroups < 1 || workgroups > 65535 || iters < 1) return PRISM_ERR_INVALID_ARG;
    return launch_probe_mfma((float*)sink, workgroups, iters, stream) == hipSuccess ? PRISM_OK : PRISM_ERR_HIP;
}

prism_status_t prism_diag_set_cu_count(int32_t cus) {
    if (cus < 0 || cus > 65535) return PRISM_ERR_INVALID_ARG;
    g_cus_forced.store(cus);
    return PRISM_OK;
}

int32_t prism_diag_cu_count(void) { return (int32_t)cu_count(); }

const char* prism_status_string(prism_status_t status) {
    switch (status) {
        case PRISM_OK: return "ok";
        case PRISM_ERR_INVALID_ARG: return "invalid argument";
        case PRISM_ERR_UNSUPPORTED: return "unsupported dtype, path or shape";
        case PRISM_ERR_WORKSPACE: return "workspace missing or too small";
        case PRISM_ERR_HIP: return "HIP runtime error";
        default: return "unknown status";
    }
}

int32_t prism_version(void) { return 200; }

}  // extern "C"
