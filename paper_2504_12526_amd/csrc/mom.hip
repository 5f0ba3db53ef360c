// libmom: C ABI over the gfx950 kernels of the MOM prefill hot path (see include/mom.h).
//
// Host side: argument validation, the mini-sequence driver (Algorithm 1, else-branch), the
// last-token LM head launch and the KV offload copies.  Nothing here allocates or synchronises.
// The only state is what mom_init resolves per device (compute-unit count, address of the static
// workspace) and the two testing overrides of mom_debug_force_gemm_form / mom_debug_force_pipeline.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>
#include <type_traits>

#include "mom.h"
#include "mom_gemm_schedule.h"
#include "mom_gemm.hip.inc"
#include "mom_gemv.hip.inc"
#include "mom_probe.hip.inc"

// Workspace of mom_mlp_prefill_static: one copy per device, held from the moment the library is
// loaded on a device until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress; the device address it yields (kept per device in g_dev) is what kernels get.
static __device__ __align__(256) unsigned char scratch[MOM_STATIC_WORKSPACE_BYTES];

namespace {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline bool overlaps(const void* a, size_t na, const void* b, size_t nb) {
    if (na == 0 || nb == 0) return false;
    uintptr_t a0 = reinterpret_cast<uintptr_t>(a), b0 = reinterpret_cast<uintptr_t>(b);
    return a0 < b0 + nb && b0 < a0 + na;
}

inline int64_t effective_chunk(int64_t S, int64_t mini_seq) {
    return (mini_seq <= 0 || mini_seq > S) ? S : mini_seq;
}

int validate_mlp(const void* x, const void* wg, const void* wu, const void* wd, int64_t S, int64_t H,
                 int64_t I, int64_t mini_seq, const void* out, const void* ws, size_t ws_bytes) {
    if (S < 0 || H <= 0 || I <= 0 || mini_seq < 0) return MOM_ERR_SHAPE;
    if ((H % 32) != 0 || (I % 32) != 0) return MOM_ERR_SHAPE;
    if (S > (int64_t)0x7fffff00 || H > (1 << 20) || I > (1 << 20)) return MOM_ERR_SHAPE;
    if (S == 0) return MOM_OK;
    if (!x || !wg || !wu || !wd || !out || !ws) return MOM_ERR_NULL;
    if (!aligned16(x) || !aligned16(wg) || !aligned16(wu) || !aligned16(wd) || !aligned16(out) ||
        !aligned16(ws))
        return MOM_ERR_ALIGN;
    const size_t need = mom_mlp_workspace_bytes(S, H, I, mini_seq);
    if (ws_bytes < need) return MOM_ERR_WORKSPACE;
    const size_t xb = (size_t)S * H * 2, wb = (size_t)H * I * 2;
    const void* ins[4] = {x, wg, wu, wd};
    const size_t inb[4] = {xb, wb, wb, wb};
    for (int i = 0; i < 4; ++i)
        if (overlaps(out, xb, ins[i], inb[i]) || overlaps(ws, need, ins[i], inb[i])) return MOM_ERR_ALIAS;
    if (overlaps(out, xb, ws, need)) return MOM_ERR_ALIAS;
    return MOM_OK;
}

// Per-device data, resolved once per device (by mom_init or by the first call that needs it) with
// that device current.
constexpr int kMaxDevices = 64;
struct DeviceInfo {
    std::atomic<int> cus{0};                 // compute units, 0 = not resolved yet
    std::atomic<void*> static_ws{nullptr};   // device address of this device's copy of `scratch`
};
DeviceInfo g_dev[kMaxDevices];

// Gate/up tiles of 96 columns beside those of 128: a column of the narrow tile costs 7 % more (measured over
// whole rounds), and the mix has to save this much of the modelled time before it is used.
constexpr int kGateUpNarrowPerMille = 1070;
constexpr int kGateUpMixMinGainPerMille = 15;

// Testing overrides (mom_debug_force_gemm_form / mom_debug_force_pipeline); 0 = the library chooses.
std::atomic<int> g_force_edge{0}, g_force_slots{0}, g_force_width{0}, g_force_pipeline{0};

DeviceInfo* current_device_info() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    return &g_dev[dev];
}

// Compute units of the current device, or 0 on error.
int compute_units() {
    DeviceInfo* d = current_device_info();
    if (!d) return 0;
    int cus = d->cus.load(std::memory_order_relaxed);
    if (cus > 0) return cus;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) return 0;
    d->cus.store(cus, std::memory_order_relaxed);
    return cus;
}

// Device address of the current device's copy of `scratch`, or nullptr on error.
void* static_workspace() {
    DeviceInfo* d = current_device_info();
    if (!d) return nullptr;
    void* p = d->static_ws.load(std::memory_order_acquire);
    if (p) return p;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
        (void)hipGetLastError();
        return nullptr;
    }
    d->static_ws.store(p, std::memory_order_release);
    return p;
}

// MOM_OK if the n bytes at p are page-locked host memory known to the HIP runtime.  Pageable memory
// would make hipMemcpyAsync stage the copy and block the calling thread, which the contract of the
// KV calls ("only enqueue") excludes.
int check_pinned_host(const void* p, size_t n) {
    const unsigned char* b = static_cast<const unsigned char*>(p);
    const unsigned char* ends[2] = {b, b + (n ? n - 1 : 0)};
    for (const unsigned char* q : ends) {
        hipPointerAttribute_t at;
        if (hipPointerGetAttributes(&at, q) != hipSuccess) {
            (void)hipGetLastError();          // an unknown pointer must not poison the next HIP call
            return MOM_ERR_HOST;
        }
        if (at.type != hipMemoryTypeHost) return MOM_ERR_HOST;
    }
    return MOM_OK;
}

// The tile grid of `a` (M, N set) for tiles of `edge` token rows staging `width` weight rows; false if it
// is empty or too large (tile numbers are 32-bit in the kernels).
template <int EPI>
bool set_tile_grid(momk::GemmArgs& a, int edge, int width) {
    const int tile_n = (EPI == momk::EPI_GATEUP) ? width / 2 : width;
    a.group_m = momk::kGroupM;
    a.tiles_m = (a.M + edge - 1) / edge;
    a.tiles_n = (a.N + tile_n - 1) / tile_n;
    const int64_t t = (int64_t)a.tiles_m * a.tiles_n;
    if (t <= 0 || t > (int64_t)0x1fffffff) return false;
    a.tiles_per_xcd = (int)((t + 7) / 8);
    return true;
}

// One launch of gemm4_kernel<EPI, edge, slots, width> over the operands in `a` (M, N, K, ldo set).
template <int EPI>
hipError_t launch_gemm_form(momk::GemmArgs a, int edge, int slots, int width, hipStream_t st) {
    if (!set_tile_grid<EPI>(a, edge, width)) return hipErrorInvalidValue;
    const dim3 grid((unsigned)(a.tiles_per_xcd * 8)), block(momk::k4Threads);
#define MOM_LAUNCH4(E, S, W) hipLaunchKernelGGL((momk::gemm4_kernel<EPI, E, S, W>), grid, block, 0, st, a)
    if (edge == 256 && slots == 5) {
        if constexpr (EPI == momk::EPI_DOWN) {
            if (width == 256) MOM_LAUNCH4(256, 5, 256);
            else if (width == 224) MOM_LAUNCH4(256, 5, 224);
            else if (width == 192) MOM_LAUNCH4(256, 5, 192);
            else if (width == 160) MOM_LAUNCH4(256, 5, 160);
            else if (width == 128) MOM_LAUNCH4(256, 5, 128);
            else return hipErrorInvalidValue;
        } else {
            if (width == 256) MOM_LAUNCH4(256, 5, 256);
            else if (width == 192) MOM_LAUNCH4(256, 5, 192);
            else return hipErrorInvalidValue;
        }
    }
    else if (edge == 128 && slots == 5 && width == 128) MOM_LAUNCH4(128, 5, 128);
    else if (edge == 128 && slots == 10 && width == 128) MOM_LAUNCH4(128, 10, 128);
    else if (edge == 64 && slots == 5 && width == 64) MOM_LAUNCH4(64, 5, 64);
    else if (edge == 64 && slots == 10 && width == 64) MOM_LAUNCH4(64, 10, 64);
    else if (edge == 64 && slots == 20 && width == 64) MOM_LAUNCH4(64, 20, 64);
    else return hipErrorInvalidValue;
#undef MOM_LAUNCH4
    return hipGetLastError();
}

template <int EPI>
hipError_t launch_gemm(const unsigned short* X, const unsigned short* W0, const unsigned short* W1,
                       unsigned short* O, int M, int N, int K, hipStream_t st, bool never_small = false) {
    momk::GemmArgs a;
    a.X = X; a.W0 = W0; a.W1 = W1; a.O = O;
    a.M = M; a.N = N; a.K = K; a.ldo = N;
    // tiles of a launch with `tile` token rows and `cols` output columns per tile
    auto tiles_of = [&](int tile, int cols) { return (int64_t)((M + tile - 1) / tile) * ((N + cols - 1) / cols); };
    const int gu = (EPI == momk::EPI_GATEUP) ? 2 : 1;        // weight rows staged per output column
    if (tiles_of(momk::kBM, momk::kBW / gu) > (int64_t)0x1fffffff) return hipErrorInvalidValue;
    // All forms give identical bits (every output element sees the same MFMA sequence over k), so the
    // choice is free.  Tile edge and ring depth: 256-tiles unless they would leave a quarter or more of
    // the CUs without work; then 128-tiles, or 64-tiles when even those fill less than half of the CUs;
    // the small tiles get a deeper ring the fewer workgroups a CU has to hide latency with.
    // Down projection with 256-row tiles: 256, 224, 192, 160 or 128 weight rows per tile, whichever needs
    // the least time in rounds of the CUs (rounds x width, a narrower tile charged more per column for the
    // token fragments it shares among fewer MFMAs, a partly filled last round less than a whole one): 3584
    // output columns with 32 token tiles are 1.75 rounds of 256-wide tiles on 256 CUs but exactly 2 rounds
    // of 224-wide ones, and the 128 full-size tiles of a 2048-row mini-sequence at 4096 columns are one
    // round of 256 tiles 128 wide.
    // Gate/up with 256-row tiles: the first columns in tiles of 128 columns, the rest in tiles of 96, in one
    // launch of the two-width kernel, where the same model says that saves time: 14336 columns with 12 token
    // tiles are 1344 tiles = 5.25 rounds, but 64 x 128 + 64 x 96 columns are three rounds of each width.
    // mom_debug_force_gemm_form overrides the choice (for tests, which need every form on shapes of
    // every size).
    const int cus = compute_units();
    if (cus <= 0) return hipErrorInvalidDevice;
    int edge = 256, slots = 0, width = 256;
    int64_t narrow_tiles_n = 0;          // gate/up: column tiles of the narrow width behind the wide ones
    const int force = g_force_edge.load(std::memory_order_relaxed);
    if (force) {
        edge = force;
        width = edge;
        const int fw = g_force_width.load(std::memory_order_relaxed);
        if (edge == 256 && fw && (EPI == momk::EPI_DOWN || fw == 192)) width = fw;
        slots = g_force_slots.load(std::memory_order_relaxed);
    } else {
        // Rounds of the CUs a launch of `tiles` tiles takes, in 1/1000.  A last round that fills only part of the
        // CUs is not as dear as a whole one: the chip is power-limited and clocks the busy CUs higher (measured:
        // a round on a quarter / half / three quarters of the CUs takes about 0.55 / 0.8 / 0.8-0.9 of a full one).
        auto rounds_pm = [&](int64_t tiles) {
            const int64_t full = tiles / cus, rem = tiles % cus;
            return full * 1000 + (rem ? 500 + 500 * rem / cus : 0);
        };
        // time in units of 1e-6 of a 256 x 256 tile per column: rounds x width x (1 + what the narrower tile costs per column)
        auto down_cost = [&](int w) {
            static const int per_mille[5] = {1000, 1020, 1070, 1170, 1310};     // 256, 224, 192, 160, 128 (measured)
            return rounds_pm(tiles_of(256, w)) * w * per_mille[(256 - w) / 32];
        };
        int64_t best = 0;
        if (EPI == momk::EPI_DOWN && !never_small)       // (beside a chip-filling gate/up kernel: full-size tiles, however few)
            for (int w : {256, 224, 192, 160, 128}) {
                const int64_t cost = down_cost(w);
                if (best == 0 || cost < best) { best = cost; width = w; }
            }
        const int64_t t256 = tiles_of(256, width / gu);
        if (!never_small && t256 * 4 <= (int64_t)cus * 3) {     // even so a quarter or more of the CUs without work
            edge = (tiles_of(128, 128 / gu) * 2 <= cus) ? 64 : 128;
            width = edge;
        } else if (EPI == momk::EPI_GATEUP) {
            // b column tiles of 96 behind a of 128: a = ceil((N - 96 b) / 128); time = rounds x columns per tile
            const int64_t tm = (M + 255) / 256;
            auto cost = [&](int64_t b) {
                const int64_t rest = (int64_t)N - 96 * b;
                const int64_t wide = rest > 0 ? (rest + 127) / 128 : 0;
                return rounds_pm(tm * wide) * 128 * 1000 + rounds_pm(tm * b) * 96 * kGateUpNarrowPerMille;
            };
            const int64_t plain = cost(0);
            int64_t best_cost = plain;
            for (int64_t b = 1; b <= ((int64_t)N + 95) / 96; ++b) {
                const int64_t c = cost(b);
                if (c < best_cost && c * 1000 <= plain * (1000 - kGateUpMixMinGainPerMille)) { best_cost = c; narrow_tiles_n = b; }
            }
        }
    }
    if (edge == 256) slots = 5;
    else if (slots == 0) {
        const int64_t t = tiles_of(edge, edge / gu);
        slots = (edge == 128) ? (t <= cus ? 10 : 5) : (t <= cus ? 20 : (t <= 2 * (int64_t)cus ? 10 : 5));
    }
    if constexpr (EPI == momk::EPI_GATEUP) {
        if (narrow_tiles_n > 0) {
            const int64_t rest = (int64_t)N - 96 * narrow_tiles_n;
            const int wide_cols = rest > 0 ? (int)((rest + 127) / 128) * 128 : 0;     // columns [0, wide_cols) in wide tiles
            if (wide_cols >= N) return launch_gemm_form<EPI>(a, 256, 5, 256, st);
            momk::GemmArgs2 p;
            p.narrow = a;
            p.narrow.W0 = W0 + (size_t)wide_cols * K;
            p.narrow.W1 = W1 + (size_t)wide_cols * K;
            p.narrow.O = O + wide_cols;
            p.narrow.N = N - wide_cols;
            if (wide_cols == 0) return launch_gemm_form<EPI>(p.narrow, 256, 5, 192, st);
            p.wide = a;
            p.wide.N = wide_cols;
            if (!set_tile_grid<EPI>(p.wide, 256, 256) || !set_tile_grid<EPI>(p.narrow, 256, 192)) return hipErrorInvalidValue;
            const int64_t wgs = 8 * ((int64_t)p.wide.tiles_per_xcd + p.narrow.tiles_per_xcd);
            if (wgs > (int64_t)0x7fffffff) return hipErrorInvalidValue;
            hipLaunchKernelGGL((momk::gemm4_two_width_kernel<EPI, 192>), dim3((unsigned)wgs), dim3(momk::k4Threads), 0, st, p);
            return hipGetLastError();
        }
    }
    return launch_gemm_form<EPI>(a, edge, slots, width, st);
}

template <int MODE>
hipError_t launch_gemv(const unsigned short* x, const unsigned short* Wa, const unsigned short* Wb, void* y,
                       int64_t R, int64_t K, hipStream_t st) {
    // Wavefronts per workgroup, batches per prefetch step and resident workgroups per CU, as measured on the
    // Llama-3-8B shapes (sweep over 2..16 wavefronts, 1..4 batches, 1..16 workgroups per CU):
    //   LM head  V x 4096     4 wavefronts, 1 batch, 2 per CU   (8 wavefronts per CU, each looping over row groups)
    //   gate/up  2 x I x 4096 2 wavefronts, 2 batches, 16 per CU
    //   down     H x 14336    8 wavefronts, 1 batch, 4 per CU   (the workgroup shares one 28 KiB copy of h in LDS)
    constexpr int WAVES = (MODE == momk::MODE_LOGITS) ? 4 : (MODE == momk::MODE_GATEUP ? 2 : 8);
    constexpr int U = (MODE == momk::MODE_GATEUP) ? 2 : 1;
    constexpr int PER_CU = (MODE == momk::MODE_LOGITS) ? 2 : (MODE == momk::MODE_GATEUP ? 16 : 4);
    const int cus = compute_units();
    if (cus <= 0) return hipErrorInvalidDevice;
    const int64_t groups = (R + momk::gemv_rows_per_group(MODE) - 1) / momk::gemv_rows_per_group(MODE);
    int64_t blocks = (groups + WAVES - 1) / WAVES;
    if (blocks > (int64_t)cus * PER_CU) blocks = (int64_t)cus * PER_CU;
    hipLaunchKernelGGL((momk::gemv_kernel<MODE, WAVES, U>), dim3((unsigned)blocks), dim3(WAVES * 64), (size_t)K * 2, st,
                       x, Wa, Wb, y, (int)R, (int)K);
    return hipGetLastError();
}

int mlp_driver(const void* x, const void* wg, const void* wu, const void* wd, int64_t S, int64_t H,
               int64_t I, int64_t mini_seq, void* out, void* ws, size_t ws_bytes, void* stream,
               void** events, int64_t n_events) {
    int rc = validate_mlp(x, wg, wu, wd, S, H, I, mini_seq, out, ws, ws_bytes);
    if (rc != MOM_OK || S == 0) return rc;
    const int64_t C = effective_chunk(S, mini_seq);
    const int64_t n = (S + C - 1) / C;
    if (events && n_events < 1 + 2 * n) return MOM_ERR_SHAPE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const unsigned short* xs = static_cast<const unsigned short*>(x);
    unsigned short* os = static_cast<unsigned short*>(out);
    unsigned short* w = static_cast<unsigned short*>(ws);
    if (events && hipEventRecord(static_cast<hipEvent_t>(events[0]), st) != hipSuccess) return MOM_ERR_HIP;
    // Algorithm 1, else-branch: O_i = MLP(A_i) for each mini-sequence, O_i written at its rows of O.
    for (int64_t c = 0; c < n; ++c) {
        const int64_t r0 = c * C;
        const int rows = (int)((r0 + C <= S) ? C : (S - r0));
        if (launch_gemm<momk::EPI_GATEUP>(xs + r0 * H, static_cast<const unsigned short*>(wg),
                                          static_cast<const unsigned short*>(wu), w, rows, (int)I, (int)H,
                                          st) != hipSuccess)
            return MOM_ERR_HIP;
        if (events && hipEventRecord(static_cast<hipEvent_t>(events[1 + 2 * c]), st) != hipSuccess)
            return MOM_ERR_HIP;
        if (launch_gemm<momk::EPI_DOWN>(w, static_cast<const unsigned short*>(wd), nullptr, os + r0 * H, rows,
                                        (int)H, (int)I, st) != hipSuccess)
            return MOM_ERR_HIP;
        if (events && hipEventRecord(static_cast<hipEvent_t>(events[2 + 2 * c]), st) != hipSuccess)
            return MOM_ERR_HIP;
    }
    return MOM_OK;
}

// The same loop on two streams with two workspace halves: the down projection of mini-sequence c
// (stream B) runs beside the gate/up projection of mini-sequence c+1 (stream A), so that the CUs
// one kernel's last, partly filled round of tiles leaves idle take tiles of the other.
//   A: [wait D(c-2)]  gate/up(c) -> half c%2   record G(c)
//   B:  wait G(c)     down(c)   <- half c%2    record D(c)
// ev[0..1] = G of even/odd c, ev[2..3] = D of even/odd c.
int mlp_pipelined(const void* x, const void* wg, const void* wu, const void* wd, int64_t S, int64_t H, int64_t I,
                  int64_t mini_seq, void* out, void* ws, size_t ws_bytes, hipStream_t sa, hipStream_t sb,
                  hipEvent_t* ev) {
    const int64_t C = effective_chunk(S, mini_seq);
    const int64_t n = (S + C - 1) / C;
    const unsigned short* xs = static_cast<const unsigned short*>(x);
    unsigned short* os = static_cast<unsigned short*>(out);
    unsigned short* half[2] = {static_cast<unsigned short*>(ws), static_cast<unsigned short*>(ws) + (size_t)C * I};
    (void)ws_bytes;
    // B starts after everything already enqueued on A (the inputs)
    if (hipEventRecord(ev[2], sa) != hipSuccess || hipStreamWaitEvent(sb, ev[2], 0) != hipSuccess) return MOM_ERR_HIP;
    for (int64_t c = 0; c < n; ++c) {
        const int64_t r0 = c * C;
        const int rows = (int)((r0 + C <= S) ? C : (S - r0));
        const int h = (int)(c & 1);
        if (c >= 2 && hipStreamWaitEvent(sa, ev[2 + h], 0) != hipSuccess) return MOM_ERR_HIP;
        // gate/up(c) is held until down(c-1) has been handed to the device: its few, long tiles must
        // get their CUs before the many tiles of this kernel take the whole chip for a round
        if (c >= 1 && hipStreamWaitEvent(sa, ev[4], 0) != hipSuccess) return MOM_ERR_HIP;
        if (launch_gemm<momk::EPI_GATEUP>(xs + r0 * H, static_cast<const unsigned short*>(wg),
                                          static_cast<const unsigned short*>(wu), half[h], rows, (int)I, (int)H,
                                          sa) != hipSuccess)
            return MOM_ERR_HIP;
        if (hipEventRecord(ev[h], sa) != hipSuccess || hipStreamWaitEvent(sb, ev[h], 0) != hipSuccess)
            return MOM_ERR_HIP;
        if (hipEventRecord(ev[4], sb) != hipSuccess) return MOM_ERR_HIP;
        // beside a gate/up kernel that fills the chip, full-size tiles are the efficient form for the
        // down projection however few they are; the last one runs alone and follows the usual rule
        const bool beside_big = c + 1 < n;
        if (launch_gemm<momk::EPI_DOWN>(half[h], static_cast<const unsigned short*>(wd), nullptr, os + r0 * H, rows,
                                        (int)H, (int)I, sb, beside_big) != hipSuccess)
            return MOM_ERR_HIP;
        if (hipEventRecord(ev[2 + h], sb) != hipSuccess) return MOM_ERR_HIP;
    }
    // A continues after the last down projection: the caller synchronises A only
    if (hipStreamWaitEvent(sa, ev[2 + (int)((n - 1) & 1)], 0) != hipSuccess) return MOM_ERR_HIP;
    return MOM_OK;
}

}  // namespace

extern "C" {

const char* mom_status_string(int status) {
    switch (status) {
        case MOM_OK: return "ok";
        case MOM_ERR_NULL: return "null pointer";
        case MOM_ERR_SHAPE: return "bad shape (H and I must be positive multiples of 32)";
        case MOM_ERR_ALIGN: return "pointer not 16-byte aligned";
        case MOM_ERR_ALIAS: return "output or workspace overlaps an input";
        case MOM_ERR_WORKSPACE: return "workspace too small";
        case MOM_ERR_HIP: return "HIP runtime error";
        case MOM_ERR_HOST: return "host pointer is not page-locked memory of the HIP runtime";
        default: return "unknown status";
    }
}

int mom_init(void) {
    if (compute_units() <= 0) return MOM_ERR_HIP;
    if (!static_workspace()) return MOM_ERR_HIP;
    return MOM_OK;
}

int mom_debug_force_gemm_form(int tile_edge, int ring_slots, int tile_width) {
    const bool wok = tile_width == 0 || (tile_edge == 256 && (tile_width == 256 || tile_width == 224 || tile_width == 192 ||
                                                              tile_width == 160 || tile_width == 128));
    const bool ok = wok && ((tile_edge == 0 && ring_slots == 0) ||
                    (tile_edge == 256 && (ring_slots == 0 || ring_slots == 5)) ||
                    (tile_edge == 128 && (ring_slots == 0 || ring_slots == 5 || ring_slots == 10)) ||
                    (tile_edge == 64 && (ring_slots == 0 || ring_slots == 5 || ring_slots == 10 || ring_slots == 20)));
    if (!ok) return MOM_ERR_SHAPE;
    g_force_width.store(tile_width, std::memory_order_relaxed);
    g_force_slots.store(ring_slots, std::memory_order_relaxed);
    g_force_edge.store(tile_edge, std::memory_order_relaxed);
    return MOM_OK;
}

int mom_debug_mfma_probe(const void* a_bf16, size_t a_bytes, const void* b_bf16, size_t b_bytes, int64_t iters,
                         int workgroups, int order, float* sink, void* stream) {
    if (!a_bf16 || !b_bf16 || !sink) return MOM_ERR_NULL;
    if (!aligned16(a_bf16) || !aligned16(b_bf16) || !aligned16(sink)) return MOM_ERR_ALIGN;
    if (a_bytes < 16 || b_bytes < 16 || a_bytes / 16 > 0x7fffffffu || b_bytes / 16 > 0x7fffffffu || iters < 0 ||
        workgroups <= 0 || workgroups > (1 << 20) || (order != 0 && order != 1))
        return MOM_ERR_SHAPE;
    const dim3 grid((unsigned)workgroups), block(momk::kProbeThreads);
    const momk::u32x4* a = static_cast<const momk::u32x4*>(a_bf16);
    const momk::u32x4* b = static_cast<const momk::u32x4*>(b_bf16);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (order == 0)
        hipLaunchKernelGGL(momk::mfma_probe_kernel<0>, grid, block, 0, st, a, (unsigned)(a_bytes / 16), b,
                           (unsigned)(b_bytes / 16), (long long)iters, sink);
    else
        hipLaunchKernelGGL(momk::mfma_probe_kernel<1>, grid, block, 0, st, a, (unsigned)(a_bytes / 16), b,
                           (unsigned)(b_bytes / 16), (long long)iters, sink);
    return hipGetLastError() == hipSuccess ? MOM_OK : MOM_ERR_HIP;
}

int mom_debug_force_pipeline(int on) {
    g_force_pipeline.store(on ? 1 : 0, std::memory_order_relaxed);
    return MOM_OK;
}

size_t mom_mlp_workspace_bytes(int64_t S, int64_t H, int64_t I, int64_t mini_seq) {
    if (S <= 0 || H <= 0 || I <= 0 || mini_seq < 0) return 0;
    return (size_t)effective_chunk(S, mini_seq) * (size_t)I * 2;
}

int mom_mlp_prefill(const void* x, const void* W_gate, const void* W_up, const void* W_down, int64_t S,
                    int64_t H, int64_t I, int64_t mini_seq, void* out, void* workspace,
                    size_t workspace_bytes, void* stream) {
    return mlp_driver(x, W_gate, W_up, W_down, S, H, I, mini_seq, out, workspace, workspace_bytes, stream,
                      nullptr, 0);
}

int mom_mlp_prefill_static(const void* x, const void* W_gate, const void* W_up, const void* W_down, int64_t S,
                           int64_t H, int64_t I, int64_t mini_seq, void* out, void* stream) {
    if (S < 0 || H <= 0 || I <= 0 || mini_seq < 0) return MOM_ERR_SHAPE;
    if (S == 0) return validate_mlp(x, W_gate, W_up, W_down, S, H, I, mini_seq, out, nullptr, 0);
    const size_t need = mom_mlp_workspace_bytes(S, H, I, mini_seq);
    if (need > (size_t)MOM_STATIC_WORKSPACE_BYTES) return MOM_ERR_WORKSPACE;
    void* ws = static_workspace();
    if (!ws) return MOM_ERR_HIP;
    return mlp_driver(x, W_gate, W_up, W_down, S, H, I, mini_seq, out, ws, (size_t)MOM_STATIC_WORKSPACE_BYTES, stream,
                      nullptr, 0);
}

size_t mom_mlp_pipelined_workspace_bytes(int64_t S, int64_t H, int64_t I, int64_t mini_seq) {
    const size_t one = mom_mlp_workspace_bytes(S, H, I, mini_seq);
    if (one == 0) return 0;
    const int64_t C = effective_chunk(S, mini_seq);
    return (S + C - 1) / C > 1 ? 2 * one : one;
}

int mom_mlp_prefill_pipelined(const void* x, const void* W_gate, const void* W_up, const void* W_down, int64_t S,
                              int64_t H, int64_t I, int64_t mini_seq, void* out, void* workspace,
                              size_t workspace_bytes, void* stream, void* stream2, void** events,
                              int64_t n_events) {
    int rc = validate_mlp(x, W_gate, W_up, W_down, S, H, I, mini_seq, out, workspace, workspace_bytes);
    if (rc != MOM_OK || S == 0) return rc;
    const size_t need = mom_mlp_pipelined_workspace_bytes(S, H, I, mini_seq);
    if (workspace_bytes < need) return MOM_ERR_WORKSPACE;
    const void* ins[4] = {x, W_gate, W_up, W_down};
    const size_t xb = (size_t)S * H * 2, wb = (size_t)H * I * 2;
    const size_t inb[4] = {xb, wb, wb, wb};
    for (int i = 0; i < 4; ++i)
        if (overlaps(workspace, need, ins[i], inb[i])) return MOM_ERR_ALIAS;
    if (overlaps(out, xb, workspace, need)) return MOM_ERR_ALIAS;
    const int64_t C = effective_chunk(S, mini_seq);
    if ((S + C - 1) / C == 1)      // a single mini-sequence: nothing to overlap
        return mlp_driver(x, W_gate, W_up, W_down, S, H, I, mini_seq, out, workspace, workspace_bytes, stream,
                          nullptr, 0);
    if (!events) return MOM_ERR_NULL;
    if (n_events < 5) return MOM_ERR_SHAPE;
    hipEvent_t ev[5];
    for (int i = 0; i < 5; ++i) {
        if (!events[i]) return MOM_ERR_NULL;
        ev[i] = static_cast<hipEvent_t>(events[i]);
    }
    // The two-stream schedule pays (measured) when the down projection of a mini-sequence leaves at least
    // half of the CUs idle, the gate/up kernel beside it is one that fills the chip with 256-tiles, and the
    // single round of long down tiles (K = I) does not outlast that kernel on the remaining CUs by more than
    // half.  Otherwise this is the plain loop.  mom_debug_force_pipeline forces the schedule (for tests,
    // which need it on shapes of every size).
    const int cus = compute_units();
    if (cus <= 0) return MOM_ERR_HIP;
    const int64_t tm = (C + momk::kBM - 1) / momk::kBM;
    const int64_t tiles_dn = tm * ((H + momk::kBW - 1) / momk::kBW);
    const int64_t tiles_gu = tm * ((I + momk::kBW / 2 - 1) / (momk::kBW / 2));
    const int64_t cus_left = cus - tiles_dn > 0 ? cus - tiles_dn : 1;
    const bool pays = 2 * tiles_dn <= cus && tiles_gu * 4 > (int64_t)cus * 3 &&
                      2 * I <= 3 * ((tiles_gu + cus_left - 1) / cus_left) * H;
    if (!g_force_pipeline.load(std::memory_order_relaxed) && !pays)
        return mlp_driver(x, W_gate, W_up, W_down, S, H, I, mini_seq, out, workspace, workspace_bytes, stream,
                          nullptr, 0);
    return mlp_pipelined(x, W_gate, W_up, W_down, S, H, I, mini_seq, out, workspace, workspace_bytes,
                         static_cast<hipStream_t>(stream), static_cast<hipStream_t>(stream2), ev);
}

int mom_mlp_prefill_events(const void* x, const void* W_gate, const void* W_up, const void* W_down,
                           int64_t S, int64_t H, int64_t I, int64_t mini_seq, void* out, void* workspace,
                           size_t workspace_bytes, void* stream, void** events, int64_t n_events) {
    if (!events) return MOM_ERR_NULL;
    return mlp_driver(x, W_gate, W_up, W_down, S, H, I, mini_seq, out, workspace, workspace_bytes, stream,
                      events, n_events);
}

int mom_lmhead_last(const void* x_last, const void* W_lm, int64_t V, float* logits, int64_t H, void* stream) {
    if (V < 0 || H <= 0 || (H % 32) != 0 || H > momk::kGemvMaxK || V > (int64_t)0x7fffff00) return MOM_ERR_SHAPE;
    if (V == 0) return MOM_OK;
    if (!x_last || !W_lm || !logits) return MOM_ERR_NULL;
    if (!aligned16(x_last) || !aligned16(W_lm) || !aligned16(logits)) return MOM_ERR_ALIGN;
    if (overlaps(logits, (size_t)V * 4, x_last, (size_t)H * 2) ||
        overlaps(logits, (size_t)V * 4, W_lm, (size_t)V * H * 2))
        return MOM_ERR_ALIAS;
    return launch_gemv<momk::MODE_LOGITS>(static_cast<const unsigned short*>(x_last),
                                          static_cast<const unsigned short*>(W_lm), nullptr, logits, V, H,
                                          static_cast<hipStream_t>(stream)) == hipSuccess ? MOM_OK : MOM_ERR_HIP;
}

int mom_mlp_last(const void* x_last, const void* W_gate, const void* W_up, const void* W_down, int64_t H,
                 int64_t I, void* out_last, void* workspace, size_t workspace_bytes, void* stream) {
    if (H <= 0 || I <= 0 || (H % 32) != 0 || (I % 32) != 0 || H > momk::kGemvMaxK || I > momk::kGemvMaxK)
        return MOM_ERR_SHAPE;
    if (!x_last || !W_gate || !W_up || !W_down || !out_last || !workspace) return MOM_ERR_NULL;
    if (!aligned16(x_last) || !aligned16(W_gate) || !aligned16(W_up) || !aligned16(W_down) ||
        !aligned16(out_last) || !aligned16(workspace))
        return MOM_ERR_ALIGN;
    const size_t need = (size_t)I * 2, hb = (size_t)H * 2, wb = (size_t)H * I * 2;
    if (workspace_bytes < need) return MOM_ERR_WORKSPACE;
    const void* ins[4] = {x_last, W_gate, W_up, W_down};
    const size_t inb[4] = {hb, wb, wb, wb};
    for (int i = 0; i < 4; ++i)
        if (overlaps(out_last, hb, ins[i], inb[i]) || overlaps(workspace, need, ins[i], inb[i])) return MOM_ERR_ALIAS;
    if (overlaps(out_last, hb, workspace, need)) return MOM_ERR_ALIAS;
    hipStream_t st = static_cast<hipStream_t>(stream);
    // h = silu(x Wg^T) .* (x Wu^T)  ->  workspace [I] bf16 ;  out = h Wd^T -> [H] bf16
    if (launch_gemv<momk::MODE_GATEUP>(static_cast<const unsigned short*>(x_last),
                                       static_cast<const unsigned short*>(W_gate),
                                       static_cast<const unsigned short*>(W_up), workspace, I, H, st) != hipSuccess)
        return MOM_ERR_HIP;
    if (launch_gemv<momk::MODE_DOWN>(static_cast<const unsigned short*>(workspace),
                                     static_cast<const unsigned short*>(W_down), nullptr, out_last, H, I,
                                     st) != hipSuccess)
        return MOM_ERR_HIP;
    return MOM_OK;
}

int mom_kv_offload(const void* k, const void* v, void* pinned_host, void* stream, size_t bytes_each,
                   void* producer_stream, void* order_event, void* done_event) {
    if (bytes_each != 0 && (!k || !v || !pinned_host)) return MOM_ERR_NULL;
    if (producer_stream && !order_event) return MOM_ERR_NULL;
    if (bytes_each != 0) {
        const int rc = check_pinned_host(pinned_host, 2 * bytes_each);
        if (rc != MOM_OK) return rc;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (order_event) {
        // producer_stream may be NULL here: that is the default stream, which does not order itself
        // against a non-blocking side stream
        hipEvent_t ev = static_cast<hipEvent_t>(order_event);
        if (hipEventRecord(ev, static_cast<hipStream_t>(producer_stream)) != hipSuccess) return MOM_ERR_HIP;
        if (hipStreamWaitEvent(st, ev, 0) != hipSuccess) return MOM_ERR_HIP;
    }
    if (bytes_each != 0) {
        unsigned char* dst = static_cast<unsigned char*>(pinned_host);
        if (hipMemcpyAsync(dst, k, bytes_each, hipMemcpyDeviceToHost, st) != hipSuccess) return MOM_ERR_HIP;
        if (hipMemcpyAsync(dst + bytes_each, v, bytes_each, hipMemcpyDeviceToHost, st) != hipSuccess)
            return MOM_ERR_HIP;
    }
    if (done_event && hipEventRecord(static_cast<hipEvent_t>(done_event), st) != hipSuccess) return MOM_ERR_HIP;
    return MOM_OK;
}

int mom_kv_reload(const void* pinned_host, void* k, void* v, void* stream, size_t bytes_each, void* done_event) {
    if (bytes_each != 0 && (!k || !v || !pinned_host)) return MOM_ERR_NULL;
    if (bytes_each != 0) {
        const int rc = check_pinned_host(pinned_host, 2 * bytes_each);
        if (rc != MOM_OK) return rc;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (bytes_each != 0) {
        const unsigned char* src = static_cast<const unsigned char*>(pinned_host);
        if (hipMemcpyAsync(k, src, bytes_each, hipMemcpyHostToDevice, st) != hipSuccess) return MOM_ERR_HIP;
        if (hipMemcpyAsync(v, src + bytes_each, bytes_each, hipMemcpyHostToDevice, st) != hipSuccess)
            return MOM_ERR_HIP;
    }
    if (done_event && hipEventRecord(static_cast<hipEvent_t>(done_event), st) != hipSuccess) return MOM_ERR_HIP;
    return MOM_OK;
}

}  // extern "C"
