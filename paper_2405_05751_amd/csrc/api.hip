// C ABI of the rmsnl library: argument checks, variant choice, workspace, launch.
#include "../../include/rmsnl.h"
#include "common.hpp"

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <mutex>
#include <tuple>
#include <vector>

using namespace rmsnl;

namespace {

constexpr size_t kDefaultWorkspace = size_t(64) << 20;   // partials + counters, per device
constexpr int kMaxDevices = 16;

thread_local char tl_error[512] = "";
thread_local rl_variant tl_last_variant = RL_AUTO;
thread_local int tl_last_plan[3] = {0, 0, 0};

std::mutex g_mu;
bool g_env_read = false;
rl_variant g_variant = RL_AUTO;
int g_n_tile = 0, g_k_split = 0;
unsigned long long* g_trace = nullptr;
int g_trace_groups = 0;
struct Workspace { void* ptr; size_t bytes; bool owned; };
Workspace g_ws[kMaxDevices] = {};
Workspace g_lent[kMaxDevices] = {};

// launch shapes found by rl_autotune, by (M, K, N, dtype, gated)
struct Tuned { rl_variant variant; int n_tile, k_split; };
typedef std::tuple<int, int, int, int, int> TuneKey;
std::map<TuneKey, Tuned> g_tuned;
// sequence splits found by rl_autotune_qknorm, by (B H, S, D, dtype)
std::map<std::tuple<int64_t, int64_t, int, int>, int> g_tuned_qk;

rl_status fail(rl_status st, const char* fmt, const char* a = "", const char* b = "")
{
    snprintf(tl_error, sizeof tl_error, fmt, a, b);
    return st;
}

void read_env_locked()
{
    if (g_env_read) return;
    g_env_read = true;
    const char* e = getenv("RL_VARIANT");
    if (!e) return;
    if (!strcmp(e, "gemv")) g_variant = RL_GEMV_SPLITK;
    else if (!strcmp(e, "skinny")) g_variant = RL_MFMA_SKINNY;
    else if (!strcmp(e, "tile")) g_variant = RL_MFMA_TILE;
    else if (!strcmp(e, "tile_pre")) g_variant = RL_MFMA_TILE_PRE;
    else if (!strcmp(e, "naive")) g_variant = RL_NAIVE;
    else if (!strcmp(e, "f32")) g_variant = RL_MFMA_F32;
    else g_variant = RL_AUTO;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

rl_status check_dims(int64_t M, int64_t K, int64_t N, rl_dtype dt)
{
    if (dt != RL_F16 && dt != RL_BF16 && dt != RL_F32) return fail(RL_ERR_INVALID_ARG, "unknown dtype");
    const int64_t lim = int64_t(1) << 31;
    if (M < 1 || K < 1 || N < 1 || M >= lim || K >= lim || N >= lim)
        return fail(RL_ERR_INVALID_ARG, "M, K, N must be in [1, 2^31)");
    return RL_OK;
}

constexpr size_t kMaxOwnWorkspace = size_t(4) << 30;

// Workspace for the current device: the lent buffer if there is one, else the library's own.  The
// library's own buffer is replaced by a larger one (at least twice the size) when a call needs
// more.  The old one is kept until the process ends: a graph captured earlier still points into
// it.  Nothing is allocated while `stream` is being captured.
rl_status get_workspace(size_t need, hipStream_t stream, Workspace* out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(RL_ERR_HIP, "hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices) return fail(RL_ERR_UNSUPPORTED, "device index out of range");
    std::lock_guard<std::mutex> lk(g_mu);
    if (g_lent[dev].ptr) {
        if (g_lent[dev].bytes < need + kHeadBytes) return fail(RL_ERR_WORKSPACE, "lent workspace too small");
        *out = g_lent[dev];
        return RL_OK;
    }
    if (!g_ws[dev].ptr || g_ws[dev].bytes < need + kHeadBytes) {
        size_t want = std::max(kDefaultWorkspace, (need + kHeadBytes + 0xfffff) & ~size_t(0xfffff));
        if (want > kMaxOwnWorkspace)
            return fail(RL_ERR_WORKSPACE, "shape needs more workspace than the library allocates; lend one with rl_set_workspace");
        want = std::min(kMaxOwnWorkspace, std::max(want, 2 * g_ws[dev].bytes));
        hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
        e = hipStreamIsCapturing(stream, &cap);
        if (e != hipSuccess) return fail(RL_ERR_HIP, "hipStreamIsCapturing: %s", hipGetErrorString(e));
        if (cap != hipStreamCaptureStatusNone)
            return fail(RL_ERR_WORKSPACE, "the workspace cannot grow during stream capture: run the shape once before, or lend a workspace");
        void* p = nullptr;
        e = hipMalloc(&p, want);
        if (e != hipSuccess) return fail(RL_ERR_HIP, "hipMalloc(workspace): %s", hipGetErrorString(e));
        e = hipMemset(p, 0, kCounterBytes);              // synchronous, once per allocation
        if (e != hipSuccess) { (void)hipFree(p); return fail(RL_ERR_HIP, "hipMemset(workspace): %s", hipGetErrorString(e)); }
        g_ws[dev] = Workspace{p, want, true};            // (a smaller predecessor stays allocated)
    }
    *out = g_ws[dev];
    return RL_OK;
}

// layout: [arrival counters | partial sums of squares | partial B]
void carve(const Workspace& ws, Problem& p)
{
    char* base = static_cast<char*>(ws.ptr);
    p.ws_counter = reinterpret_cast<unsigned*>(base);
    p.ws_sumsq = reinterpret_cast<float*>(base + kCounterBytes);
    p.ws_partial = reinterpret_cast<float*>(base + kHeadBytes);
}

// ---- the workspace of the entry point that allocates nothing: a file-scope device array.  Every
// device the library runs on holds its own copy, at its own address, until the process ends; the
// array's name is only a host-side handle, and the address the kernels get is looked up once per
// device.  Same layout as every other workspace (see carve()).
constexpr size_t kScratchBytes = size_t(8) << 20;
}  // namespace
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
namespace {
void* g_scratch[kMaxDevices] = {};       // device address of the current device's copy, once looked up

__global__ void scratch_clear_kernel(unsigned* p, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

rl_status get_scratch(hipStream_t s, Workspace* out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(RL_ERR_HIP, "hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices) return fail(RL_ERR_UNSUPPORTED, "device index out of range");
    std::lock_guard<std::mutex> lk(g_mu);
    if (!g_scratch[dev]) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) return fail(RL_ERR_HIP, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
        // the arrival counters must start at zero (the kernels leave them at zero after every call); a
        // fill kernel, not a memset, so that a caller may capture this first call into a graph
        const int n = int(kCounterBytes / sizeof(unsigned));
        scratch_clear_kernel<<<(n + 255) / 256, 256, 0, s>>>(static_cast<unsigned*>(ptr), n);
        e = hipGetLastError();
        if (e != hipSuccess) return fail(RL_ERR_HIP, "clearing the scratch counters: %s", hipGetErrorString(e));
        g_scratch[dev] = ptr;
    }
    *out = Workspace{g_scratch[dev], kScratchBytes, false};
    return RL_OK;
}

rl_variant choose_auto(const Problem& p)
{
    if (p.dt == F32) return RL_MFMA_F32;     // what it cannot run (gated, odd sizes) falls through to the plain kernel
    if (p.N % 8 != 0 || p.K % 8 != 0) return RL_NAIVE;
    if (p.gated && p.N % 16 != 0) return RL_NAIVE;
    // one row: the GEMV kernel is ahead by 2 to 8 % while W needs a deep split over K to fill the chip
    // (measured at N <= 8192; at N = 11008, 13824, 14336 the matrix-core kernel is 10-17 % ahead).  Two
    // to four rows: the GEMV kernel's shorter chain of dependent steps wins while W is small (2 x 2048 x
    // 2048: 6.5 against 8.8 us, 4 x 2048 x 2048: 7.6 against 8.8 us; 2 x 3072 x 3072: 12.9 against 11.3 us).
    if (p.M == 1 && p.N < 10240) return RL_GEMV_SPLITK;
    if (p.M <= 4 && double(p.K) * p.N <= 6.0e6) return RL_GEMV_SPLITK;
    if (p.M <= 64) return RL_MFMA_SKINNY;
    // Above 64 rows the skinny kernel runs one row block per 64 rows in the same launch; every row
    // block pulls its own copy of W into its compute unit (from L2 after the first), so it wins
    // while (row blocks) x K x N is small and loses to the tile kernels beyond about 1.4e8, earlier
    // for wide W (measured: 128x4096x6144 27 against 31 us, 512x4096x4096 37 against 43 us,
    // 1024x2048x2048 22 against 37 us; 768x1024x8192 41 against 37 us, 128x8192x10240 70 against
    // 59 us, 256x4096x28672 131 against 81 us).  With two row blocks the wide-W limit does not apply
    // (128x4096x14336 41 against 47 us, 128x8192x8192 44 against 53 us, 128x7168x7168 40 against 45 us).
    const int row_blocks = (p.M + 63) / 64;
    if (p.M <= 1024 && double(row_blocks) * p.K * p.N <= (p.N <= 6144 || row_blocks == 2 ? 1.4e8 : 0.9e8)) return RL_MFMA_SKINNY;
    return RL_MFMA_TILE;
}

// The fused tile kernel repeats the X-hat conversion in every one of its N / 256 workgroup
// columns and cannot split K; writing X-hat once (4 M K bytes of traffic) and running the product
// on it, split over K when its tiles are few, measured faster at every tile-sized shape tried
// (M 65 to 8192, N 2048 to 28672), so the fused tile kernel is what runs when the workspace has no
// room for X-hat.
bool prefers_two_kernels(const Problem& p)
{
    return p.fused != 0 || tile_pre_workspace_bytes(p) != 0;   // the plain product: only where it is split over K
}

// one attempt at one variant; hipErrorInvalidValue = the variant cannot run the shape
// fixed: the one workspace this call may use (nothing is allocated), or null for the library's own or the lent one
hipError_t launch_variant(rl_variant v, Problem& p, hipStream_t s, const char** why, rl_status* ws_status,
                          const Workspace* fixed = nullptr)
{
    *ws_status = RL_OK;
    size_t need = 0;
    if (v == RL_GEMV_SPLITK) need = gemv_workspace_bytes(p);
    else if (v == RL_MFMA_SKINNY) need = skinny_workspace_bytes(p);
    else if (v == RL_MFMA_TILE_PRE) need = tile_pre_workspace_bytes(p);
    else if (v == RL_MFMA_F32) need = f32_workspace_bytes(p);
    p.ws_partial = nullptr; p.ws_sumsq = nullptr; p.ws_counter = nullptr;
    if (need) {
        Workspace ws;
        if (fixed) {
            ws = *fixed;
            *ws_status = ws.bytes >= need + kHeadBytes ? RL_OK
                : fail(RL_ERR_WORKSPACE, "the shape needs more workspace than this call's buffer holds (the scratch array of rmsnorm_linear_noalloc: 8 MiB in all)");
        } else {
            *ws_status = get_workspace(need, s, &ws);
        }
        if (*ws_status != RL_OK) return hipErrorUnknown;
        carve(ws, p);
    }
    switch (v) {
    case RL_GEMV_SPLITK: return launch_gemv(p, s, why);
    case RL_MFMA_SKINNY: return launch_skinny(p, s, why);
    case RL_MFMA_TILE:   return launch_tile(p, s, why);
    case RL_MFMA_TILE_PRE: return launch_tile_pre(p, s, why);
    case RL_NAIVE:       return launch_naive(p, s, why);
    case RL_MFMA_F32:    return launch_f32(p, s, why);
    default:             return hipErrorInvalidValue;
    }
}

// opts: this call's variant and launch shape instead of the process-wide settings (or null)
struct CallOpts { rl_variant variant; int n_tile, k_split; };

rl_status run(Problem& p, void* stream, const Workspace* fixed = nullptr, const CallOpts* opts = nullptr)
{
    rl_variant forced;
    Tuned tuned{RL_AUTO, 0, 0};
    {
        std::lock_guard<std::mutex> lk(g_mu);
        read_env_locked();
        forced = opts ? opts->variant : g_variant;
        p.n_tile = opts ? opts->n_tile : g_n_tile;
        p.k_split = opts ? opts->k_split : g_k_split;
        p.trace = g_trace;
        p.trace_groups = g_trace_groups;
        if (forced == RL_AUTO) {
            auto it = g_tuned.find(TuneKey(p.M, p.K, p.N, int(p.dt), p.gated | (p.gate_group ? 2 : 0)));
            if (it != g_tuned.end() && p.fused) tuned = it->second;
        }
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    tl_last_plan[0] = tl_last_plan[1] = tl_last_plan[2] = 0;
    p.plan = tl_last_plan;
    rl_variant order[6];
    int n_order = 0;
    if (forced != RL_AUTO) {
        order[n_order++] = forced;
    } else {
        p.n_tile = 0;                      // tuning overrides apply to a forced variant only
        p.k_split = 0;
        if (tuned.variant != RL_AUTO) order[n_order++] = tuned.variant;    // with its launch shape, see below
        rl_variant first = choose_auto(p);
        if (first == RL_MFMA_TILE && prefers_two_kernels(p)) order[n_order++] = RL_MFMA_TILE_PRE;
        order[n_order++] = first;
        if (first == RL_MFMA_SKINNY && p.M > 64) order[n_order++] = RL_MFMA_TILE;   // e.g. no room for the split
        if (first != RL_NAIVE) order[n_order++] = RL_NAIVE;
    }
    const char* why = "variant cannot run this shape";
    for (int i = 0; i < n_order; ++i) {
        rl_variant v = order[i];
        why = "variant cannot run this shape";
        if (forced == RL_AUTO) {
            const bool use_tuned = (i == 0 && tuned.variant != RL_AUTO);
            p.n_tile = use_tuned ? tuned.n_tile : 0;
            p.k_split = use_tuned ? tuned.k_split : 0;
        }
        rl_status ws_status;
        hipError_t e = launch_variant(v, p, s, &why, &ws_status, fixed);
        if (ws_status != RL_OK) {
            // the two-kernel form is an optimisation: without room for it the fused kernel runs; a
            // tuned launch shape likewise gives way to the built-in one
            if (forced == RL_AUTO && ws_status == RL_ERR_WORKSPACE &&
                (v == RL_MFMA_TILE_PRE || (i == 0 && tuned.variant != RL_AUTO))) continue;
            return ws_status;
        }
        if (e == hipSuccess) { tl_last_variant = v; return RL_OK; }
        if (e != hipErrorInvalidValue) return fail(RL_ERR_HIP, "kernel launch: %s", hipGetErrorString(e));
        (void)hipGetLastError();
    }
    return fail(RL_ERR_UNSUPPORTED, "%s", why);
}

}  // namespace

extern "C" {

rl_status rmsnorm_linear(const void* X, const void* g, const void* W, float eps, void* Y,
                         int64_t M, int64_t K, int64_t N, rl_dtype dt, void* stream)
{
    if (!X || !g || !W || !Y) return fail(RL_ERR_INVALID_ARG, "null pointer");
    if (rl_status st = check_dims(M, K, N, dt)) return st;
    if (!std::isfinite(eps) || eps < 0.f) return fail(RL_ERR_INVALID_ARG, "eps must be finite and >= 0");
    if (!aligned16(X) || !aligned16(g) || !aligned16(W) || !aligned16(Y))
        return fail(RL_ERR_INVALID_ARG, "pointers must be 16-byte aligned");
    Problem p{};
    p.X = X; p.g = g; p.W = W; p.Y = Y;
    p.M = int(M); p.K = int(K); p.N = int(N);
    p.eps = eps; p.fused = 1; p.dt = DType(dt);
    return run(p, stream);
}

rl_status rmsnorm_linear_noalloc(const void* X, const void* g, const void* W, float eps, void* Y,
                                 int64_t M, int64_t K, int64_t N, rl_dtype dt, void* stream)
{
    if (!X || !g || !W || !Y) return fail(RL_ERR_INVALID_ARG, "null pointer");
    if (rl_status st = check_dims(M, K, N, dt)) return st;
    if (!std::isfinite(eps) || eps < 0.f) return fail(RL_ERR_INVALID_ARG, "eps must be finite and >= 0");
    if (!aligned16(X) || !aligned16(g) || !aligned16(W) || !aligned16(Y))
        return fail(RL_ERR_INVALID_ARG, "pointers must be 16-byte aligned");
    Workspace ws;
    if (rl_status st = get_scratch(static_cast<hipStream_t>(stream), &ws)) return st;
    Problem p{};
    p.X = X; p.g = g; p.W = W; p.Y = Y;
    p.M = int(M); p.K = int(K); p.N = int(N);
    p.eps = eps; p.fused = 1; p.dt = DType(dt);
    return run(p, stream, &ws);
}

size_t rl_noalloc_scratch_bytes(void) { return kScratchBytes; }

// the options of an _ex call as the launchers' (n_tile, k_split) pair, which means something else per variant
static rl_status translate_opts(const rl_launch_opts* o, CallOpts* c, Workspace* ws, bool* has_ws)
{
    *has_ws = false;
    c->variant = RL_AUTO; c->n_tile = 0; c->k_split = 0;
    if (!o) return RL_OK;
    if (o->struct_size != sizeof(rl_launch_opts)) return fail(RL_ERR_INVALID_ARG, "rl_launch_opts.struct_size must be sizeof(rl_launch_opts)");
    if (o->variant < RL_AUTO || o->variant > RL_MFMA_F32) return fail(RL_ERR_INVALID_ARG, "unknown variant");
    if (o->columns < 0 || o->slabs < 0 || o->waves < 0 || o->rem_slabs < 0)
        return fail(RL_ERR_INVALID_ARG, "launch options must be >= 0");
    c->variant = o->variant;
    switch (o->variant) {
    case RL_GEMV_SPLITK: case RL_MFMA_SKINNY: case RL_MFMA_F32: c->n_tile = o->columns; c->k_split = o->slabs; break;
    case RL_MFMA_TILE: c->n_tile = o->columns; c->k_split = o->waves; break;
    case RL_MFMA_TILE_PRE:
        if (o->slabs) { c->n_tile = 1; c->k_split = o->slabs; }
        else if (o->rem_slabs) { c->n_tile = 2; c->k_split = o->rem_slabs; }
        break;
    default: break;
    }
    if (o->workspace) {
        if (!aligned16(o->workspace) || o->workspace_bytes <= kHeadBytes)
            return fail(RL_ERR_INVALID_ARG, "workspace must be 16-byte aligned and larger than 1280 KiB");
        *ws = Workspace{o->workspace, o->workspace_bytes, false};
        *has_ws = true;
    }
    return RL_OK;
}

rl_status rmsnorm_linear_ex(const void* X, const void* g, const void* W, float eps, void* Y,
                            int64_t M, int64_t K, int64_t N, rl_dtype dt, const rl_launch_opts* opts, void* stream)
{
    if (!X || !g || !W || !Y) return fail(RL_ERR_INVALID_ARG, "null pointer");
    if (rl_status st = check_dims(M, K, N, dt)) return st;
    if (!std::isfinite(eps) || eps < 0.f) return fail(RL_ERR_INVALID_ARG, "eps must be finite and >= 0");
    if (!aligned16(X) || !aligned16(g) || !aligned16(W) || !aligned16(Y))
        return fail(RL_ERR_INVALID_ARG, "pointers must be 16-byte aligned");
    CallOpts c; Workspace ws; bool has_ws;
    if (rl_status st = translate_opts(opts, &c, &ws, &has_ws)) return st;
    Problem p{};
    p.X = X; p.g = g; p.W = W; p.Y = Y;
    p.M = int(M); p.K = int(K); p.N = int(N);
    p.eps = eps; p.fused = 1; p.dt = DType(dt);
    return run(p, stream, has_ws ? &ws : nullptr, opts ? &c : nullptr);
}

rl_status rmsnorm_gated_mlp_ex(const void* X, const void* g, const void* W, float eps, void* Y,
                               int64_t M, int64_t K, int64_t H, rl_dtype dt, int interleaved,
                               const rl_launch_opts* opts, void* stream)
{
    if (!X || !g || !W || !Y) return fail(RL_ERR_INVALID_ARG, "null pointer");
    if (H < 1 || H >= (int64_t(1) << 30)) return fail(RL_ERR_INVALID_ARG, "H must be in [1, 2^30)");
    if (interleaved && H % 64 != 0) return fail(RL_ERR_INVALID_ARG, "the interleaved layout needs H % 64 == 0");
    if (rl_status st = check_dims(M, K, 2 * H, dt)) return st;
    if (!std::isfinite(eps) || eps < 0.f) return fail(RL_ERR_INVALID_ARG, "eps must be finite and >= 0");
    if (!aligned16(X) || !aligned16(g) || !aligned16(W) || !aligned16(Y))
        return fail(RL_ERR_INVALID_ARG, "pointers must be 16-byte aligned");
    CallOpts c; Workspace ws; bool has_ws;
    if (rl_status st = translate_opts(opts, &c, &ws, &has_ws)) return st;
    Problem p{};
    p.X = X; p.g = g; p.W = W; p.Y = Y;
    p.M = int(M); p.K = int(K); p.N = int(2 * H);
    p.eps = eps; p.fused = 1; p.gated = 1; p.gate_group = interleaved ? 64 : 0; p.dt = DType(dt);
    return run(p, stream, has_ws ? &ws : nullptr, opts ? &c : nullptr);
}

rl_status rl_last_launch(rl_variant* variant, int* columns, int* slabs, int* workgroups)
{
    if (!variant || !columns || !slabs || !workgroups) return fail(RL_ERR_INVALID_ARG, "null pointer");
    *variant = tl_last_variant; *columns = tl_last_plan[0]; *slabs = tl_last_plan[1]; *workgroups = tl_last_plan[2];
    return RL_OK;
}

rl_status rmsnorm_gated_mlp(const void* X, const void* g, const void* W, float eps, void* Y,
                            int64_t M, int64_t K, int64_t H, rl_dtype dt, void* stream)
{
    if (!X || !g || !W || !Y) return fail(RL_ERR_INVALID_ARG, "null pointer");
    if (H < 1 || H >= (int64_t(1) << 30)) return fail(RL_ERR_INVALID_ARG, "H must be in [1, 2^30)");
    if (rl_status st = check_dims(M, K, 2 * H, dt)) return st;
    if (!std::isfinite(eps) || eps < 0.f) return fail(RL_ERR_INVALID_ARG, "eps must be finite and >= 0");
    if (!aligned16(X) || !aligned16(g) || !aligned16(W) || !aligned16(Y))
        return fail(RL_ERR_INVALID_ARG, "pointers must be 16-byte aligned");
    Problem p{};
    p.X = X; p.g = g; p.W = W; p.Y = Y;
    p.M = int(M); p.K = int(K); p.N = int(2 * H);
    p.eps = eps; p.fused = 1; p.gated = 1; p.dt = DType(dt);
    return run(p, stream);
}

rl_status rmsnorm_gated_mlp_interleaved(const void* X, const void* g, const void* Wi, float eps, void* Y,
                                        int64_t M, int64_t K, int64_t H, rl_dtype dt, void* stream)
{
    if (!X || !g || !Wi || !Y) return fail(RL_ERR_INVALID_ARG, "null pointer");
    if (H < 1 || H >= (int64_t(1) << 30)) return fail(RL_ERR_INVALID_ARG, "H must be in [1, 2^30)");
    if (H % 64 != 0) return fail(RL_ERR_INVALID_ARG, "the interleaved layout needs H % 64 == 0");
    if (rl_status st = check_dims(M, K, 2 * H, dt)) return st;
    if (!std::isfinite(eps) || eps < 0.f) return fail(RL_ERR_INVALID_ARG, "eps must be finite and >= 0");
    if (!aligned16(X) || !aligned16(g) || !aligned16(Wi) || !aligned16(Y))
        return fail(RL_ERR_INVALID_ARG, "pointers must be 16-byte aligned");
    Problem p{};
    p.X = X; p.g = g; p.W = Wi; p.Y = Y;
    p.M = int(M); p.K = int(K); p.N = int(2 * H);
    p.eps = eps; p.fused = 1; p.gated = 1; p.gate_group = 64; p.dt = DType(dt);
    return run(p, stream);
}

rl_status rl_interleave_gate_up(const void* W, void* Wi, int64_t K, int64_t H, rl_dtype dt, void* stream)
{
    if (!W || !Wi) return fail(RL_ERR_INVALID_ARG, "null pointer");
    if (W == Wi) return fail(RL_ERR_INVALID_ARG, "W and Wi must be different buffers");
    if (H < 1 || H >= (int64_t(1) << 30)) return fail(RL_ERR_INVALID_ARG, "H must be in [1, 2^30)");
    if (H % 64 != 0) return fail(RL_ERR_INVALID_ARG, "the interleaved layout needs H % 64 == 0");
    if (rl_status st = check_dims(1, K, 2 * H, dt)) return st;
    if (!aligned16(W) || !aligned16(Wi)) return fail(RL_ERR_INVALID_ARG, "pointers must be 16-byte aligned");
    hipError_t e = launch_interleave_gate_up(W, Wi, K, int(H), DType(dt), static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(RL_ERR_HIP, "kernel launch: %s", hipGetErrorString(e));
    return RL_OK;
}

rl_status silu_mul(const void* Z, void* Y, int64_t M, int64_t H, rl_dtype dt, void* stream)
{
    if (!Z || !Y) return fail(RL_ERR_INVALID_ARG, "null pointer");
    if (H < 1 || H >= (int64_t(1) << 30)) return fail(RL_ERR_INVALID_ARG, "H must be in [1, 2^30)");
    if (rl_status st = check_dims(M, 1, 2 * H, dt)) return st;
    if (M > 65535) return fail(RL_ERR_UNSUPPORTED, "silu_mul supports M <= 65535");
    if (!aligned16(Z) || !aligned16(Y)) return fail(RL_ERR_INVALID_ARG, "pointers must be 16-byte aligned");
    hipError_t e = launch_silu_mul(Z, Y, int(M), int(H), DType(dt), static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(RL_ERR_HIP, "kernel launch: %s", hipGetErrorString(e));
    return RL_OK;
}

rl_status matmul(const void* A, const void* W, void* Y, int64_t M, int64_t K, int64_t N, rl_dtype dt,
                 void* stream)
{
    if (!A || !W || !Y) return fail(RL_ERR_INVALID_ARG, "null pointer");
    if (rl_status st = check_dims(M, K, N, dt)) return st;
    if (!aligned16(A) || !aligned16(W) || !aligned16(Y))
        return fail(RL_ERR_INVALID_ARG, "pointers must be 16-byte aligned");
    Problem p{};
    p.X = A; p.g = nullptr; p.W = W; p.Y = Y;
    p.M = int(M); p.K = int(K); p.N = int(N);
    p.eps = 0.f; p.fused = 0; p.dt = DType(dt);
    return run(p, stream);
}

rl_status rmsnorm(const void* X, const void* g, float eps, void* Xn, int64_t M, int64_t K, rl_dtype dt,
                  void* stream)
{
    if (!X || !g || !Xn) return fail(RL_ERR_INVALID_ARG, "null pointer");
    if (rl_status st = check_dims(M, K, 1, dt)) return st;
    if (!std::isfinite(eps) || eps < 0.f) return fail(RL_ERR_INVALID_ARG, "eps must be finite and >= 0");
    if (!aligned16(X) || !aligned16(g) || !aligned16(Xn))
        return fail(RL_ERR_INVALID_ARG, "pointers must be 16-byte aligned");
    hipError_t e = launch_rmsnorm(X, g, eps, Xn, int(M), int(K), DType(dt), static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(RL_ERR_HIP, "kernel launch: %s", hipGetErrorString(e));
    return RL_OK;
}

// The tuner's core: every launch shape the library has for the call, timed on `stream` while the
// launches rotate through n_w copies of W (one copy: W is timed as it lies in the caches).
static rl_status autotune_core(const void* X, const void* g, const void* const* Ws, int n_w, float eps, void* Y,
                               int64_t M, int64_t K, int64_t N, rl_dtype dt, int gated, int interleaved, int reps,
                               void* stream, float* best_us)
{
    if (!X || !g || !Ws || !Y || n_w < 1) return fail(RL_ERR_INVALID_ARG, "null pointer");
    for (int i = 0; i < n_w; ++i)
        if (!Ws[i] || !aligned16(Ws[i])) return fail(RL_ERR_INVALID_ARG, "every copy of W must be a 16-byte aligned device pointer");
    if (rl_status st = check_dims(M, K, N, dt)) return st;
    if (gated && (N % 2)) return fail(RL_ERR_INVALID_ARG, "the gated block needs an even N (= 2H)");
    if (interleaved && (!gated || (N / 2) % 64)) return fail(RL_ERR_INVALID_ARG, "the interleaved layout is the gated block's, H % 64 == 0");
    if (reps < 1 || reps > 1000) return fail(RL_ERR_INVALID_ARG, "reps must be in [1, 1000]");
    if (!std::isfinite(eps) || eps < 0.f) return fail(RL_ERR_INVALID_ARG, "eps must be finite and >= 0");
    if (!aligned16(X) || !aligned16(g) || !aligned16(Y))
        return fail(RL_ERR_INVALID_ARG, "pointers must be 16-byte aligned");
    Problem base{};
    base.X = X; base.g = g; base.W = Ws[0]; base.Y = Y;
    base.M = int(M); base.K = int(K); base.N = int(N);
    base.eps = eps; base.fused = 1; base.gated = gated ? 1 : 0; base.gate_group = interleaved ? 64 : 0; base.dt = DType(dt);

    // The launch shapes worth trying, generated from the shape: (variant, n_tile, k_split); 0 = that
    // kernel's own default.  GEMV and skinny: every slab count that keeps at least one batch (run) of
    // rows per lane group (wave), at each column width; slab counts that round to the same slabs are
    // launched once.
    struct Cand { rl_variant v; int n_tile, k_split; };
    std::vector<Cand> cands;
    if (dt != RL_F32) {
        if (M <= 16)
            for (int nt : {128, 256, 512}) {
                cands.push_back({RL_GEMV_SPLITK, nt, 0});
                for (int ks = 1; ks <= 32; ++ks) cands.push_back({RL_GEMV_SPLITK, nt, ks});
            }
        if (M <= 1024)
            for (int nt : {0, 64})
                for (int ks = 1; ks <= 16; ++ks) cands.push_back({RL_MFMA_SKINNY, nt, ks});
        if (M > 16)
            for (int shape : {256, 512})
                for (int nw : {4, 8}) cands.push_back({RL_MFMA_TILE, shape, nw});
        if (M > 64)                        // two-kernel form: the library's own K split, none, 2 to 16 slabs
            for (int ks : {0, 1, 2, 4, 8, 16}) cands.push_back({RL_MFMA_TILE_PRE, ks ? 1 : 0, ks});
    }
    if (dt == RL_F32)
        for (int ks = 0; ks <= 16; ++ks) cands.push_back({RL_MFMA_F32, 0, ks});
    cands.push_back({RL_NAIVE, 0, 0});

    hipStream_t s = static_cast<hipStream_t>(stream);
    hipEvent_t e0 = nullptr, e1 = nullptr;
    hipError_t he = hipEventCreate(&e0);
    if (he == hipSuccess) he = hipEventCreate(&e1);
    if (he != hipSuccess) {
        if (e0) (void)hipEventDestroy(e0);
        return fail(RL_ERR_HIP, "hipEventCreate: %s", hipGetErrorString(he));
    }
    Tuned best{RL_AUTO, 0, 0};
    float best_ms = 0.f;
    rl_status result = RL_OK;
    std::vector<std::tuple<int, int, int, int>> seen;           // (variant, columns, slabs, workgroups) already timed
    int plan[3];
    for (const Cand& c : cands) {
        if (c.v == RL_NAIVE && best.variant != RL_AUTO) break;      // the fallback only if nothing else runs
        Problem p = base;
        p.n_tile = c.n_tile; p.k_split = c.k_split;
        p.plan = plan;
        const char* why = nullptr;
        rl_status ws_status;
        bool ok = true;
        for (int i = 0; i < 2 + reps && ok; ++i) {
            if (i == 2) he = hipEventRecord(e0, s);
            p.W = Ws[i % n_w];
            plan[0] = plan[1] = plan[2] = 0;
            hipError_t le = launch_variant(c.v, p, s, &why, &ws_status);
            if (ws_status != RL_OK || le == hipErrorInvalidValue) { (void)hipGetLastError(); ok = false; break; }
            if (le != hipSuccess) { result = fail(RL_ERR_HIP, "kernel launch: %s", hipGetErrorString(le)); ok = false; }
            if (i == 0) {                                           // the same launch as an earlier candidate: once is enough
                const auto key = std::make_tuple(int(c.v), plan[0], plan[1], plan[2]);
                if (plan[2] != 0 && std::find(seen.begin(), seen.end(), key) != seen.end()) { ok = false; break; }
                seen.push_back(key);
            }
        }
        if (result != RL_OK) break;
        if (!ok) continue;
        he = hipEventRecord(e1, s);
        if (he == hipSuccess) he = hipEventSynchronize(e1);
        float ms = 0.f;
        if (he == hipSuccess) he = hipEventElapsedTime(&ms, e0, e1);
        if (he != hipSuccess) { result = fail(RL_ERR_HIP, "timing: %s", hipGetErrorString(he)); break; }
        if (best.variant == RL_AUTO || ms < best_ms) { best = Tuned{c.v, c.n_tile, c.k_split}; best_ms = ms; }
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (result != RL_OK) return result;
    if (best.variant == RL_AUTO) return fail(RL_ERR_UNSUPPORTED, "no variant runs this shape");
    {
        std::lock_guard<std::mutex> lk(g_mu);
        g_tuned[TuneKey(base.M, base.K, base.N, int(base.dt), base.gated | (base.gate_group ? 2 : 0))] = best;
    }
    if (best_us) *best_us = best_ms * 1000.f / float(reps);
    return RL_OK;
}

rl_status rl_autotune(const void* X, const void* g, const void* W, float eps, void* Y,
                      int64_t M, int64_t K, int64_t N, rl_dtype dt, int gated, int reps,
                      void* stream, float* best_us)
{
    if (!W) return fail(RL_ERR_INVALID_ARG, "null pointer");
    return autotune_core(X, g, &W, 1, eps, Y, M, K, N, dt, gated, 0, reps, stream, best_us);
}

rl_status rl_autotune_rotating(const void* X, const void* g, const void* const* W_copies, int n_copies, float eps, void* Y,
                               int64_t M, int64_t K, int64_t N, rl_dtype dt, int gated, int interleaved, int reps,
                               void* stream, float* best_us)
{
    if (n_copies < 1 || n_copies > 4096) return fail(RL_ERR_INVALID_ARG, "n_copies must be in [1, 4096]");
    return autotune_core(X, g, W_copies, n_copies, eps, Y, M, K, N, dt, gated, interleaved, reps, stream, best_us);
}

rl_status rl_autotune_get(int64_t M, int64_t K, int64_t N, rl_dtype dt, int gated,
                          rl_variant* variant, int* n_tile, int* k_split)
{
    if (!variant || !n_tile || !k_split) return fail(RL_ERR_INVALID_ARG, "null pointer");
    if (rl_status st = check_dims(M, K, N, dt)) return st;
    std::lock_guard<std::mutex> lk(g_mu);
    auto it = g_tuned.find(TuneKey(int(M), int(K), int(N), int(dt), gated & 3));     // bit 1: the interleaved layout
    if (it == g_tuned.end()) { *variant = RL_AUTO; *n_tile = 0; *k_split = 0; return RL_OK; }
    *variant = it->second.variant; *n_tile = it->second.n_tile; *k_split = it->second.k_split;
    return RL_OK;
}

void rl_autotune_clear(void)
{
    std::lock_guard<std::mutex> lk(g_mu);
    g_tuned.clear();
    g_tuned_qk.clear();
}

rl_status rl_ntrans(const void* X, const void* H, const void* alpha, float eps, void* Y,
                    int64_t M, int64_t D, rl_dtype dt, void* stream)
{
    if (!X || !H || !alpha || !Y) return fail(RL_ERR_INVALID_ARG, "null pointer");
    if (rl_status st = check_dims(M, D, 1, dt)) return st;
    if (!std::isfinite(eps) || eps < 0.f) return fail(RL_ERR_INVALID_ARG, "eps must be finite and >= 0");
    if (!aligned16(X) || !aligned16(H) || !aligned16(alpha) || !aligned16(Y))
        return fail(RL_ERR_INVALID_ARG, "pointers must be 16-byte aligned");
    hipError_t e = launch_ntrans(X, H, alpha, eps, Y, int(M), int(D), DType(dt), static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(RL_ERR_HIP, "kernel launch: %s", hipGetErrorString(e));
    return RL_OK;
}

static rl_status qknorm_check(const void* Q, const void* K, const void* V, const void* gq, const void* bq,
                              const void* gk, const void* bk, float eps, const void* O,
                              int64_t B, int64_t H, int64_t S, int64_t D, rl_dtype dt)
{
    if (!Q || !K || !V || !gq || !bq || !gk || !bk || !O) return fail(RL_ERR_INVALID_ARG, "null pointer");
    if (dt != RL_F16 && dt != RL_BF16 && dt != RL_F32) return fail(RL_ERR_INVALID_ARG, "unknown dtype");
    if (B < 1 || H < 1 || S < 1 || D < 1 || B * H > (int64_t(1) << 24) || S > (int64_t(1) << 22) || D > 4096)
        return fail(RL_ERR_INVALID_ARG, "need 1 <= B*H <= 2^24, 1 <= S <= 2^22, 1 <= D <= 4096");
    if (!std::isfinite(eps) || eps < 0.f) return fail(RL_ERR_INVALID_ARG, "eps must be finite and >= 0");
    for (const void* ptr : {Q, K, V, gq, bq, gk, bk, O})
        if (!aligned16(ptr)) return fail(RL_ERR_INVALID_ARG, "pointers must be 16-byte aligned");
    return RL_OK;
}

// splits: 0 = the library's rule, else that many sequence splits
static rl_status qknorm_launch(const void* Q, const void* K, const void* V, const void* gq, const void* bq,
                               const void* gk, const void* bk, float eps, void* O,
                               int64_t B, int64_t H, int64_t S, int64_t D, rl_dtype dt, int splits, hipStream_t s)
{
    float* ws = nullptr;
    unsigned* counters = nullptr;
    const size_t need = qkattn_workspace_bytes(B, H, S, D, DType(dt));
    if (need) {
        Workspace w;
        if (rl_status st = get_workspace(need, s, &w)) return st;
        counters = static_cast<unsigned*>(w.ptr);
        ws = reinterpret_cast<float*>(static_cast<char*>(w.ptr) + kHeadBytes);
    }
    hipError_t e = launch_qkattn(Q, K, V, gq, bq, gk, bk, eps, O, B, H, S, D, DType(dt), ws, counters, splits, s);
    if (e != hipSuccess) return fail(RL_ERR_HIP, "kernel launch: %s", hipGetErrorString(e));
    return RL_OK;
}

rl_status rl_qknorm_attention(const void* Q, const void* K, const void* V, const void* gq, const void* bq,
                              const void* gk, const void* bk, float eps, void* O,
                              int64_t B, int64_t H, int64_t S, int64_t D, rl_dtype dt, void* stream)
{
    if (rl_status st = qknorm_check(Q, K, V, gq, bq, gk, bk, eps, O, B, H, S, D, dt)) return st;
    int splits;
    {
        std::lock_guard<std::mutex> lk(g_mu);
        splits = g_k_split;                  // rl_set_tuning(., k_split): sequence splits of this kernel
        if (splits == 0) {
            auto it = g_tuned_qk.find(std::make_tuple(B * H, S, int(D), int(dt)));
            if (it != g_tuned_qk.end()) splits = it->second;
        }
    }
    return qknorm_launch(Q, K, V, gq, bq, gk, bk, eps, O, B, H, S, D, dt, splits, static_cast<hipStream_t>(stream));
}

rl_status rl_autotune_qknorm(const void* Q, const void* const* K_copies, const void* const* V_copies, int n_copies,
                             const void* gq, const void* bq, const void* gk, const void* bk, float eps, void* O,
                             int64_t B, int64_t H, int64_t S, int64_t D, rl_dtype dt, int reps, void* stream,
                             int* best_splits, float* best_us)
{
    if (!K_copies || !V_copies || n_copies < 1 || n_copies > 4096)
        return fail(RL_ERR_INVALID_ARG, "need 1 to 4096 copies of K and V");
    if (reps < 1 || reps > 1000) return fail(RL_ERR_INVALID_ARG, "reps must be in [1, 1000]");
    for (int i = 0; i < n_copies; ++i)
        if (rl_status st = qknorm_check(Q, K_copies[i], V_copies[i], gq, bq, gk, bk, eps, O, B, H, S, D, dt)) return st;
    if (best_splits) *best_splits = 0;
    if (best_us) *best_us = 0.f;
    const int automatic = qkattn_splits(B, H, S, D, DType(dt), 0);
    if (automatic == 0) return RL_OK;                    // the plain kernel has no launch shape to search
    // every split count that leaves at least 64 positions to a split; counts that round to the same
    // number of splits are launched once; the library's own rule goes first and wins ties
    std::vector<int> cands{0};
    std::vector<int> seen{automatic};
    for (int sp = 1; sp <= 64; ++sp) {
        const int got = qkattn_splits(B, H, S, D, DType(dt), sp);
        if (std::find(seen.begin(), seen.end(), got) != seen.end()) continue;
        seen.push_back(got);
        cands.push_back(sp);
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipEvent_t e0 = nullptr, e1 = nullptr;
    hipError_t he = hipEventCreate(&e0);
    if (he == hipSuccess) he = hipEventCreate(&e1);
    if (he != hipSuccess) {
        if (e0) (void)hipEventDestroy(e0);
        return fail(RL_ERR_HIP, "hipEventCreate: %s", hipGetErrorString(he));
    }
    int best = -1;
    float best_ms = 0.f;
    rl_status result = RL_OK;
    for (int sp : cands) {
        for (int i = 0; i < 2 + reps && result == RL_OK; ++i) {
            if (i == 2) he = hipEventRecord(e0, s);
            result = qknorm_launch(Q, K_copies[i % n_copies], V_copies[i % n_copies], gq, bq, gk, bk, eps, O, B, H, S, D, dt, sp, s);
        }
        if (result != RL_OK) break;
        if (he == hipSuccess) he = hipEventRecord(e1, s);
        if (he == hipSuccess) he = hipEventSynchronize(e1);
        float ms = 0.f;
        if (he == hipSuccess) he = hipEventElapsedTime(&ms, e0, e1);
        if (he != hipSuccess) { result = fail(RL_ERR_HIP, "timing: %s", hipGetErrorString(he)); break; }
        if (best < 0 || ms < best_ms) { best = sp; best_ms = ms; }
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (result != RL_OK) return result;
    {
        std::lock_guard<std::mutex> lk(g_mu);
        if (best > 0) g_tuned_qk[std::make_tuple(B * H, S, int(D), int(dt))] = best;
        else g_tuned_qk.erase(std::make_tuple(B * H, S, int(D), int(dt)));
    }
    if (best_splits) *best_splits = best > 0 ? qkattn_splits(B, H, S, D, DType(dt), best) : automatic;
    if (best_us) *best_us = best_ms * 1000.f / float(reps);
    return RL_OK;
}

rl_status rl_ff_rmsnorm_linear(const void* X, const void* g, const void* W, void* Y,
                               int64_t M, int64_t K, int64_t N, uint32_t p, int reordered, void* stream)
{
    if (!X || !g || !W || !Y) return fail(RL_ERR_INVALID_ARG, "null pointer");
    if (rl_status st = check_dims(M, K, N, RL_F32)) return st;
    if (M > 65535) return fail(RL_ERR_UNSUPPORTED, "the finite-field block supports M <= 65535");
    bool prime = p >= 3 && p <= 32749;
    for (uint32_t d = 2; prime && d * d <= p; ++d) prime = (p % d) != 0;
    if (!prime) return fail(RL_ERR_INVALID_ARG, "p must be a prime in [3, 32749]");
    if (K % int64_t(p) == 0) return fail(RL_ERR_INVALID_ARG, "p must not divide K (the mean needs 1/K)");
    hipError_t e = launch_ff_block(X, g, W, Y, int(M), int(K), int(N), p, reordered ? 1 : 0,
                                   static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(RL_ERR_HIP, "kernel launch: %s", hipGetErrorString(e));
    return RL_OK;
}

rl_status rl_ff_pairs(const void* X, const void* g, const void* W, void* Y, int64_t M, int64_t K, int64_t N,
                      uint32_t omega, int gated, int schedule, int slabs, void* stream)
{
    if (!X || !g || !W || !Y) return fail(RL_ERR_INVALID_ARG, "null pointer");
    if (rl_status st = check_dims(M, K, N, RL_BF16)) return st;
    if (!aligned16(X) || !aligned16(g) || !aligned16(W) || !aligned16(Y))
        return fail(RL_ERR_INVALID_ARG, "pointers must be 16-byte aligned");
    if (schedule != 0 && schedule != 1) return fail(RL_ERR_INVALID_ARG, "schedule must be 0 (reference graph) or 1 (gemv split-K kernel)");
    if (slabs < 0) return fail(RL_ERR_INVALID_ARG, "slabs must be >= 0");
    if (gated && (N % 2)) return fail(RL_ERR_INVALID_ARG, "the gated block needs an even N (= 2H)");
    if (K % int64_t(kFfP) == 0 || K % int64_t(kFfQ) == 0) return fail(RL_ERR_INVALID_ARG, "neither 227 nor 113 may divide K (the mean needs 1/K)");
    uint64_t w = omega % kFfP, t = 1;
    for (uint32_t i = 0; i < kFfQ; ++i) t = t * w % kFfP;
    if (omega == 0 || omega >= kFfP || t != 1) return fail(RL_ERR_INVALID_ARG, "omega must be a 113th root of unity of Z_227");
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (schedule == 0) {
        if (M > 65535) return fail(RL_ERR_UNSUPPORTED, "the reference evaluation supports M <= 65535");
        hipError_t e = launch_ff_pairs_ref(X, g, W, Y, int(M), int(K), int(N), omega, gated ? 1 : 0, s);
        return e == hipSuccess ? RL_OK : fail(RL_ERR_HIP, "kernel launch: %s", hipGetErrorString(e));
    }
    Problem p{};
    p.X = X; p.g = g; p.W = W; p.Y = Y;
    p.M = int(M); p.K = int(K); p.N = int(N);
    p.fused = 1; p.gated = gated ? 1 : 0; p.dt = BF16; p.n_tile = 128; p.k_split = slabs;
    tl_last_plan[0] = tl_last_plan[1] = tl_last_plan[2] = 0;
    p.plan = tl_last_plan;
    const size_t need = gemv_workspace_bytes(p);
    if (need) {
        Workspace ws;
        if (rl_status st = get_workspace(need, s, &ws)) return st;
        carve(ws, p);
    }
    const char* why = "the gemv kernel cannot run this shape";
    hipError_t e = launch_gemv_ff(p, omega, s, &why);
    if (e == hipErrorInvalidValue) { (void)hipGetLastError(); return fail(RL_ERR_UNSUPPORTED, "%s", why); }
    if (e != hipSuccess) return fail(RL_ERR_HIP, "kernel launch: %s", hipGetErrorString(e));
    tl_last_variant = RL_GEMV_SPLITK;
    return RL_OK;
}

rl_status rl_set_variant(rl_variant v)
{
    if (v < RL_AUTO || v > RL_MFMA_F32) return fail(RL_ERR_INVALID_ARG, "unknown variant");
    std::lock_guard<std::mutex> lk(g_mu);
    g_env_read = true;
    g_variant = v;
    return RL_OK;
}

rl_variant rl_get_variant(void)
{
    std::lock_guard<std::mutex> lk(g_mu);
    read_env_locked();
    return g_variant;
}

rl_variant rl_last_variant(void) { return tl_last_variant; }

rl_status rl_set_tuning(int n_tile, int k_split)
{
    if (n_tile < 0 || k_split < 0) return fail(RL_ERR_INVALID_ARG, "tuning values must be >= 0");
    std::lock_guard<std::mutex> lk(g_mu);
    g_n_tile = n_tile;
    g_k_split = k_split;
    return RL_OK;
}

rl_status rl_set_trace(void* dev_ptr, size_t bytes)
{
    if (dev_ptr && ((reinterpret_cast<uintptr_t>(dev_ptr) & 7u) || bytes < kTraceSlots * 8))
        return fail(RL_ERR_INVALID_ARG, "trace buffer must be 8-byte aligned and hold at least one workgroup");
    std::lock_guard<std::mutex> lk(g_mu);
    g_trace = static_cast<unsigned long long*>(dev_ptr);
    g_trace_groups = dev_ptr ? int(std::min<size_t>(bytes / (kTraceSlots * 8), size_t(1) << 30)) : 0;
    return RL_OK;
}

size_t rl_trace_slots(void) { return kTraceSlots; }

rl_status rl_tile_order(int64_t M, int64_t N, int64_t position, int64_t* tile_row, int64_t* tile_col)
{
    if (!tile_row || !tile_col) return fail(RL_ERR_INVALID_ARG, "null output pointer");
    if (M < 1 || N < 1) return fail(RL_ERR_INVALID_ARG, "tile order needs M, N >= 1");
    const int64_t tiles_m = (M + 255) / 256, tiles_n = (N + 255) / 256;
    if (tiles_m * tiles_n > (int64_t(1) << 24) || tiles_m > (int64_t(1) << 24) || tiles_n > (int64_t(1) << 24))
        return fail(RL_ERR_INVALID_ARG, "more than 2^24 tiles");
    if (position < 0 || position >= tiles_m * tiles_n) return fail(RL_ERR_INVALID_ARG, "position outside the launch");
    int tm = 0, tn = 0;
    tile_order_at(int(position), int(tiles_m), int(tiles_n), &tm, &tn);
    *tile_row = tm; *tile_col = tn;
    return RL_OK;
}

rl_status rl_set_workspace(void* dev_ptr, size_t bytes)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(RL_ERR_HIP, "hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices) return fail(RL_ERR_UNSUPPORTED, "device index out of range");
    if (dev_ptr && (!aligned16(dev_ptr) || bytes <= kHeadBytes))
        return fail(RL_ERR_INVALID_ARG, "workspace must be 16-byte aligned and larger than 1280 KiB");
    std::lock_guard<std::mutex> lk(g_mu);
    g_lent[dev] = Workspace{dev_ptr, dev_ptr ? bytes : 0, false};
    return RL_OK;
}

size_t rl_workspace_bytes(int64_t M, int64_t K, int64_t N, rl_dtype dt)
{
    if (check_dims(M, K, N, dt) != RL_OK) return 0;
    Problem p{};
    p.M = int(M); p.K = int(K); p.N = int(N); p.dt = DType(dt); p.fused = 1;
    rl_variant v;
    Tuned tuned{RL_AUTO, 0, 0};
    {
        std::lock_guard<std::mutex> lk(g_mu);
        read_env_locked();
        v = g_variant;
        if (v != RL_AUTO) { p.n_tile = g_n_tile; p.k_split = g_k_split; }
        else {
            auto it = g_tuned.find(TuneKey(p.M, p.K, p.N, int(p.dt), 0));
            if (it != g_tuned.end()) tuned = it->second;
        }
    }
    auto need_of = [](rl_variant var, const Problem& q) -> size_t {
        if (var == RL_GEMV_SPLITK) return gemv_workspace_bytes(q);
        if (var == RL_MFMA_SKINNY) return skinny_workspace_bytes(q);
        if (var == RL_MFMA_TILE_PRE) return tile_pre_workspace_bytes(q);
        if (var == RL_MFMA_F32) return f32_workspace_bytes(q);
        return 0;
    };
    size_t need = 0;
    if (v == RL_AUTO) {
        v = choose_auto(p);
        if (v == RL_MFMA_TILE && prefers_two_kernels(p)) v = RL_MFMA_TILE_PRE;   // optional: without it the fused kernel runs
        need = need_of(v, p);
        if (tuned.variant != RL_AUTO) {        // a shape found by rl_autotune runs first: room for whichever needs more
            Problem q = p;
            q.n_tile = tuned.n_tile; q.k_split = tuned.k_split;
            need = std::max(need, need_of(tuned.variant, q));
        }
    } else {
        need = need_of(v, p);
    }
    return need ? need + kHeadBytes : 0;
}

size_t rl_workspace_default_bytes(void) { return kDefaultWorkspace; }

rl_status rl_probe_copy(void* dst, const void* src, size_t bytes, void* stream)
{
    if (!dst || !src || bytes == 0 || bytes % 16 || !aligned16(dst) || !aligned16(src))
        return fail(RL_ERR_INVALID_ARG, "probe copy needs 16-byte aligned pointers and size");
    hipError_t e = launch_probe_copy(dst, src, bytes, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? RL_OK : fail(RL_ERR_HIP, "kernel launch: %s", hipGetErrorString(e));
}

rl_status rl_probe_read(const void* src, size_t bytes, void* sink, void* stream)
{
    if (!sink || !src || bytes == 0 || bytes % 16 || !aligned16(src))
        return fail(RL_ERR_INVALID_ARG, "probe read needs 16-byte aligned pointer and size");
    hipError_t e = launch_probe_read(src, bytes, sink, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? RL_OK : fail(RL_ERR_HIP, "kernel launch: %s", hipGetErrorString(e));
}

rl_status rl_probe_read_strips(const void* src, int64_t rows, int64_t row_bytes, int parts, void* sink, void* stream)
{
    if (!sink || !src || !aligned16(src)) return fail(RL_ERR_INVALID_ARG, "probe needs a sink and a 16-byte aligned source");
    if (rows < 1 || row_bytes < 256 || row_bytes % 256 || parts < 1 || parts > rows ||
        (rows + 256) * row_bytes >= (int64_t(1) << 31) || (row_bytes / 256) * int64_t(parts) > (int64_t(1) << 20))
        return fail(RL_ERR_INVALID_ARG, "strips probe: row_bytes a multiple of 256, 1 <= parts <= rows, (rows + 256) * row_bytes < 2^31");
    unsigned long long* trace;
    int trace_groups;
    {
        std::lock_guard<std::mutex> lk(g_mu);
        trace = g_trace; trace_groups = g_trace_groups;
    }
    hipError_t e = launch_probe_strips(src, int(rows), int(row_bytes), parts, sink, trace, trace_groups,
                                       static_cast<hipStream_t>(stream));
    return e == hipSuccess ? RL_OK : fail(RL_ERR_HIP, "kernel launch: %s", hipGetErrorString(e));
}

rl_status rl_probe_read_flat(const void* src, size_t bytes, int workgroups, void* sink, void* stream)
{
    if (!sink || !src || bytes == 0 || bytes % 16 || !aligned16(src) || workgroups < 1 || workgroups > (1 << 20))
        return fail(RL_ERR_INVALID_ARG, "flat probe needs a sink, a 16-byte aligned source and size, 1 <= workgroups <= 2^20");
    hipError_t e = launch_probe_flat(src, bytes, workgroups, sink, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? RL_OK : fail(RL_ERR_HIP, "kernel launch: %s", hipGetErrorString(e));
}

rl_status rl_probe_mfma_operands(void* sink, int iters, rl_dtype dt, int zero_operands, void* stream)
{
    if (!sink || iters < 1 || (dt != RL_F16 && dt != RL_BF16))
        return fail(RL_ERR_INVALID_ARG, "probe mfma needs a sink, iters >= 1 and a 16-bit type");
    hipError_t e = launch_probe_mfma(sink, iters, DType(dt), zero_operands != 0, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? RL_OK : fail(RL_ERR_HIP, "kernel launch: %s", hipGetErrorString(e));
}

rl_status rl_probe_mfma(void* sink, int iters, rl_dtype dt, void* stream)
{
    return rl_probe_mfma_operands(sink, iters, dt, 0, stream);
}

const char* rl_last_error(void) { return tl_error; }
const char* rl_version(void) { return "rmsnl 0.1 (gfx950)"; }

}  // extern "C"
