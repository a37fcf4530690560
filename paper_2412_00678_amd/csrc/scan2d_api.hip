// C ABI of the 2D selective scan library: argument validation, variant selection, launches.
// The operation and every argument are specified in include/scan2d.h.
#include "../../include/scan2d.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>

#include <mutex>

#include "scan2d_variants.hpp"
#include "scan2d_bwd.hpp"
#include "scan2d_elementwise.hpp"
#include "scan2d_block.hpp"
#include "scan2d_tuning.hpp"

namespace scan2d {

// ------------------------------------------------------------------ tuning overrides (see scan2d_tuning.hpp)
namespace {
TuneSlot g_tune[kTuneKinds];
std::once_flag g_tune_env_once;

void tune_read_env() {
    static const char* const names[kTuneKinds] = {"SCAN2D_FWD_VARIANT", "SCAN2D_FWD_SHARED", "SCAN2D_BWD_VARIANT"};
    for (int k = 0; k < kTuneKinds; ++k) {
        const char* e = std::getenv(names[k]);
        if (e == nullptr) continue;
        int v[kTuneMaxValues] = {0, 0, 0, 0, 0, 0};
        const int n = std::sscanf(e, "%d,%d,%d,%d,%d,%d", &v[0], &v[1], &v[2], &v[3], &v[4], &v[5]);
        if (n > 0) {
            for (int i = 0; i < kTuneMaxValues; ++i) g_tune[k].v[i].store(v[i], std::memory_order_relaxed);
            g_tune[k].n.store(n, std::memory_order_release);
        }
    }
}
}  // namespace

TuneValues tune_get(int kind) {
    std::call_once(g_tune_env_once, tune_read_env);
    TuneValues t;
    if (kind < 0 || kind >= kTuneKinds) return t;
    t.n = g_tune[kind].n.load(std::memory_order_acquire);
    for (int i = 0; i < kTuneMaxValues; ++i) t.v[i] = g_tune[kind].v[i].load(std::memory_order_relaxed);
    return t;
}

void tune_set(int kind, const int* values, int n) {
    std::call_once(g_tune_env_once, tune_read_env);
    if (kind < 0 || kind >= kTuneKinds) return;
    if (n < 0 || values == nullptr) n = 0;
    if (n > kTuneMaxValues) n = kTuneMaxValues;
    g_tune[kind].n.store(0, std::memory_order_release);
    for (int i = 0; i < kTuneMaxValues; ++i) g_tune[kind].v[i].store(i < n ? values[i] : 0, std::memory_order_relaxed);
    g_tune[kind].n.store(n, std::memory_order_release);
}

namespace {

constexpr int kMaxDevices = 64;
std::atomic<int> g_device_ok[kMaxDevices];   // 0 = unknown, 1 = gfx950, -1 = something else

int check_device() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return SCAN2D_ERR_UNSUPPORTED_DEVICE;
    if (dev < 0 || dev >= kMaxDevices) return SCAN2D_ERR_UNSUPPORTED_DEVICE;
    int st = g_device_ok[dev].load(std::memory_order_relaxed);
    if (st == 0) {
        hipDeviceProp_t prop;
        if (hipGetDeviceProperties(&prop, dev) != hipSuccess) return SCAN2D_ERR_UNSUPPORTED_DEVICE;
        st = (std::strncmp(prop.gcnArchName, "gfx950", 6) == 0) ? 1 : -1;
        g_device_ok[dev].store(st, std::memory_order_relaxed);
    }
    return st == 1 ? SCAN2D_OK : SCAN2D_ERR_UNSUPPORTED_DEVICE;
}

int check_desc(const scan2d_desc* d) {
    if (d == nullptr) return SCAN2D_ERR_NULL_POINTER;
    if (d->Bt < 1 || d->Dc < 1 || d->H < 1 || d->W < 1 || d->N < 1 || d->N > 64) return SCAN2D_ERR_BAD_SHAPE;
    if (d->dtype != SCAN2D_F32 && d->dtype != SCAN2D_BF16) return SCAN2D_ERR_BAD_DTYPE;
    if ((d->flags & ~(uint32_t)(SCAN2D_FLAG_IDENTITY_CELLS | SCAN2D_FLAG_COLUMNS_FIRST)) != 0u) return SCAN2D_ERR_BAD_FLAGS;
    // element counts must fit 63 bits, and one map's states must be addressable with 32-bit
    // lane offsets (fill_choice checks the exact span): N * H * W < 2^27 bounds it
    const double M = (double)d->Bt * d->Dc * d->H * d->W;
    const double S = (double)d->Bt * d->N * d->H * d->W;
    if (M >= 9.0e18 || S >= 9.0e18) return SCAN2D_ERR_BAD_SHAPE;
    if ((double)d->N * d->H * d->W >= 134217728.0) return SCAN2D_ERR_BAD_SHAPE;
    return SCAN2D_OK;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// ------------------------------------------------------------------ forward variant choice
struct FwdChoice {
    int LG = 0, K = 0, NW = 0, waves = 4;
    bool exact = true, fast = true, multi = false, sp = false;
    int RPB = 1;
    size_t lds_bytes = 0;
    int NG = 0, MPW = 0, panels = 0;
    bool shared = false;          // the form that computes the per-position values once per map (scan2d_fwd_shared.hpp)
    bool cf = false;              // columns first inside the kernel
    bool skew = false;            // shared form with skewed rows: lane l of a group on row t - l, no scan across the lanes
    bool tile = false;            // one workgroup per map of at most 16 x 16 positions (scan2d_fwd_tile16.hip)
    FwdKernel kernel = nullptr;
};

struct V4 { int LG, K, NW, waves; };
#define SCAN2D_X(lg, k, nw, wv) {lg, k, nw, wv},
const V4 kFwdVariants[] = {SCAN2D_FWD_VARIANTS(SCAN2D_X)};
#undef SCAN2D_X

size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

FwdKernel lookup(int dtype, int LG, int K, int NW, int waves, bool exact, bool fast, bool multi, bool sp, bool ma, bool ua) {
    return dtype == SCAN2D_BF16 ? fwd_kernel_bf16(LG, K, NW, waves, exact, fast, multi, sp, ma, ua)
                                : fwd_kernel_f32(LG, K, NW, waves, exact, fast, multi, sp, ma);
}

// rpb: rows between two barriers; 0 = decide here
// ma: the mask rows (if any) start on 4-byte boundaries
bool fill_choice(const scan2d_desc* d, int LG, int K, int NW, int waves, int rpb, bool sp, bool ma, FwdChoice* out) {
    const int slots = waves * 64 / LG;
    FwdChoice c;
    c.LG = LG; c.K = K; c.NW = NW; c.waves = waves; c.sp = sp;
    c.exact = (d->N % NW) == 0;
    c.NG = (d->N + NW - 1) / NW;
    if (c.NG > slots) return false;
    c.MPW = slots / c.NG;
    c.panels = (d->W + LG * K - 1) / (LG * K);
    c.multi = c.panels > 1;
    // unguarded loads whenever one panel covers the row (bf16 rows of odd width and mask rows off the 4-byte
    // boundaries have instantiations that shift the elements into place)
    const bool ua = d->dtype == SCAN2D_BF16 && (d->W % 2) != 0;
    c.fast = !c.multi;
    // 32-bit lane offsets span up to `slots` maps and `slots + 1` batch items of states
    const double span = (double)(slots + 1) * d->N * d->H * d->W * 4.0;
    if (span >= 2147483648.0) return false;
    c.kernel = lookup(d->dtype, LG, K, NW, waves, c.exact, c.fast, c.multi, sp, ma, ua);
    if (c.kernel == nullptr) return false;
    // LDS for the partial sums: 2 buffers x RPB rows x (threads * K) floats.  Few large maps (one
    // workgroup per CU at most) can afford 128 KB (8 rows per barrier measured 1-3 % faster than 4 there);
    // otherwise stay near 24 KB so that several workgroups fit a CU.
    const size_t row_bytes = (size_t)waves * 64 * K * sizeof(float);
    const double wgs = std::ceil((double)d->Bt * d->Dc / c.MPW);
    const size_t budget = wgs <= 256.0 ? 131072 : 24576;
    c.RPB = 1;
    if (c.NG > 1) {
        if (rpb == 1 || rpb == 2 || rpb == 4 || rpb == 8) c.RPB = rpb;
        else if (wgs <= 256.0 && 2 * 8 * row_bytes <= budget) c.RPB = 8;
        else if (2 * 4 * row_bytes <= budget) c.RPB = 4;
        else if (2 * 2 * row_bytes <= budget) c.RPB = 2;
    }
    c.lds_bytes = c.NG > 1 ? 2 * (size_t)c.RPB * row_bytes : 0;
    if (c.lds_bytes > 160 * 1024) return false;
    *out = c;
    return true;
}

// Narrow maps: one wavefront per map, its four DPP rows share the states (scan2d_fwd_small.hpp).
bool fill_small(const scan2d_desc* d, int KS, bool sp, FwdChoice* out) {
    if (d->W > 16 * KS) return false;
    int NW = 1;
    while (4 * NW < d->N) NW *= 2;
    FwdChoice c;
    c.LG = 16; c.K = KS; c.NW = NW; c.waves = 4;
    c.exact = true; c.fast = false; c.multi = false;
    c.NG = 4; c.MPW = 4; c.panels = 1; c.RPB = 1; c.lds_bytes = 0;
    c.kernel = d->dtype == SCAN2D_BF16 ? fwd_small_kernel_bf16(KS, NW, sp) : fwd_small_kernel_f32(KS, NW, sp);
    if (c.kernel == nullptr) return false;
    *out = c;
    return true;
}

// Few maps of at most 16 x 16 positions and 16 states: one workgroup per map, rows and columns as parallel scans
// (scan2d_fwd_tile16.hip).  With many maps the kernel above wins: it repeats nothing and runs four maps per workgroup.
#ifndef SCAN2D_TILE16_MAX_MAPS
#define SCAN2D_TILE16_MAX_MAPS 1024
#endif
bool fill_tile16(const scan2d_desc* d, bool sp, FwdChoice* out) {
    if (d->H > 16 || d->W > 16 || d->N > 16 || (long long)d->Bt * d->Dc > SCAN2D_TILE16_MAX_MAPS) return false;
    FwdChoice c;
    c.LG = 16; c.K = 1; c.NW = d->N; c.waves = 4; c.sp = sp;
    c.exact = true; c.fast = false; c.multi = false; c.tile = true;
    c.NG = 1; c.MPW = 1; c.panels = 1; c.RPB = 1; c.lds_bytes = 0;
    c.kernel = fwd_tile16_kernel(d->dtype, sp);
    *out = c;
    return true;
}

// The form whose lane groups share the per-position work through LDS: single panel, N = NG * NW exactly,
// whole maps per workgroup.
struct V6 { int LG, K, NW, NG, waves, RPB; };
#define SCAN2D_X(lg, k, nw, ng, wv, rpb) {lg, k, nw, ng, wv, rpb},
const V6 kFwdSharedVariants[] = {SCAN2D_FWD_SHARED_VARIANTS(SCAN2D_X)};
#undef SCAN2D_X

// skew: the tilings with skewed rows; they read whole dwords along the diagonal, so bf16 rows must have an even width
bool fill_shared(const scan2d_desc* d, int LG, int K, int NW, int waves, int RPB, bool sp, FwdChoice* out, bool cf = false, bool skew = false) {
    if (NW < 1 || LG < 16 || K < 4 || waves < 1 || RPB < 2) return false;
    if (d->N % NW != 0 || d->W > LG * K) return false;
    if (skew && (cf || (d->dtype == SCAN2D_BF16 && (d->W % 2) != 0))) return false;
    const int slots = waves * 64 / LG, NG = d->N / NW;
    if (NG > slots || slots % NG != 0) return false;
    FwdChoice c;
    c.LG = LG; c.K = K; c.NW = NW; c.waves = waves; c.sp = sp; c.RPB = RPB;
    c.exact = true; c.fast = true; c.multi = false; c.shared = true;
    c.NG = NG; c.MPW = slots / NG; c.panels = 1;
    const double span = (double)(slots + 1) * d->N * d->H * d->W * 4.0;
    if (span >= 2147483648.0) return false;
    const bool ua = d->dtype == SCAN2D_BF16 && (d->W % 2) != 0;
    c.cf = cf; c.skew = skew;
    if (skew) c.kernel = fwd_skew_kernel(d->dtype == SCAN2D_BF16, LG, K, NW, NG, waves, RPB, sp);
    else if (cf) c.kernel = d->dtype == SCAN2D_BF16 ? fwd_shared_kernel_bf16_cf(LG, K, NW, NG, waves, RPB, sp, ua)
                                               : fwd_shared_kernel_f32_cf(LG, K, NW, NG, waves, RPB, sp);
    else c.kernel = d->dtype == SCAN2D_BF16 ? fwd_shared_kernel_bf16(LG, K, NW, NG, waves, RPB, sp, ua)
                                            : fwd_shared_kernel_f32(LG, K, NW, NG, waves, RPB, sp);
    if (c.kernel == nullptr) return false;
    const size_t panel = (size_t)LG * K;
    c.lds_bytes = (2 * (size_t)c.MPW * RPB * 2 * panel + 2 * (size_t)RPB * slots * panel) * sizeof(float);
    if (c.lds_bytes > 160 * 1024) return false;
    *out = c;
    return true;
}

// VGPRs + AGPRs of the compiled forward kernels (more than 256 means one wave per SIMD), used only to rank
// variants.  The table is generated by the build from the compiler's resource-usage remarks for exactly the
// kernels that are linked into this library.
struct PlainRegs { int K, NW, b, f; };
struct SharedRegs { int bf16, LG, K, NW, NG, waves, RPB, regs; };
#include "scan2d_fwd_regs.inc"

int fwd_regs(bool bf16, int K, int NW) {
    for (const PlainRegs& r : kPlainRegs)
        if (r.K == K && r.NW == NW) return bf16 ? r.b : r.f;
    return 300;
}
int fwd_shared_regs(bool bf16, const V6& v) {
    for (const SharedRegs& r : kSharedRegs)
        if (r.bf16 == (bf16 ? 1 : 0) && r.LG == v.LG && r.K == v.K && r.NW == v.NW && r.NG == v.NG && r.waves == v.waves && r.RPB == v.RPB)
            return r.regs;
    return 300;
}

// Estimated run time (arbitrary units) of a variant, used only to rank the variants.  Calibrated
// against measurements on the benchmark shapes: instructions per workgroup row (core
// arithmetic, lane-group scans, per-position work, fixed loop overhead, LDS reduction) times
// rows, divided by the issue efficiency that the number of resident waves per SIMD allows
// (about 0.5 / 0.7 / 0.9 for 1 / 2 / 3 and more waves).
double fwd_cost(const scan2d_desc* d, const FwdChoice& c) {
    const bool bf16 = d->dtype == SCAN2D_BF16;
    const double maps = (double)d->Bt * d->Dc;
    const double wgs = std::ceil(maps / c.MPW);
    const double c_core = bf16 ? 10.5 : 8.5;
    // a lone recurrence pads its DPP wait states (16- and 32-lane scans; the wave-wide scan has enough steps of its own)
    const double c_scan = (c.LG == 64 ? 13.0 : (c.LG == 32 ? 12.0 : 9.0)) + (c.NW == 1 && c.LG != 64 ? 4.0 : 0.0);
    const double c_pos = bf16 ? 9.0 : 6.0;
    const double cols_t = std::max(1.0, (double)c.K / c.NG);
    double c_red = c.NG > 1 ? cols_t * (4.0 + 1.5 * c.NG) + 6.0 : 4.0;
    // shared-producer form: the per-position work is done once per map, every cell is summed by one thread
    double pos = c_pos * c.K;
    if (c.shared) {
        pos = (c_pos + 4.0) * c.K / c.NG + 4.0;
        c_red = (double)c.K / c.NG * (c.NG + 6.0) + 4.0;
    }
    double row = c.K * c.NW * c_core + c.NW * c_scan + pos + (c.shared ? 8.0 : 35.0) + c_red;
    if (!c.fast) row *= 1.6;
    if (c.multi) row += 8.0 * c.NW;
    // the instantiations that compute the step need one or two VGPRs more, which matters at the 256 boundary
    const V6 v6{c.LG, c.K, c.NW, c.NG, c.waves, c.RPB};
    const double regs = (c.shared ? fwd_shared_regs(bf16, v6) : fwd_regs(bf16, c.K, c.NW)) + (c.sp ? 2 : 0);
    const double occ = std::min(8.0, std::max(std::floor(512.0 / regs), c.waves / 4.0));
    double wg_cu = std::max(1.0, std::floor(occ * 4.0 / c.waves));                    // workgroups resident on a CU: registers ...
    if (c.lds_bytes > 0) wg_cu = std::min(wg_cu, std::max(1.0, std::floor(163840.0 / (double)c.lds_bytes)));   // ... and LDS
    const double res_wg = 256.0 * wg_cu;                                             // workgroups resident on the chip
    const double rounds = std::ceil(wgs / res_wg);
    double wps = std::min(std::min(occ, wg_cu * c.waves / 4.0), wgs * c.waves / 1024.0 / rounds);
    if (rounds > 1.0) wps = std::max(wps, 1.0);                                      // several rounds: SIMDs are never empty
    const double steps = (double)d->H * c.panels * row;                              // instructions of one wave
    if (wps < 1.0) return steps * 8.0;                                               // a lone wave: its own critical path
    // measured issue efficiencies: the plain kernels keep gaining up to four waves per SIMD, the shared-producer
    // kernels (fewer, longer dependent chains per row and an LDS hand-over) level off near 0.88 (256 maps of 256x256
    // bf16: one state per lane on 16 waves 124 us, two states per lane on 8 waves 133 us; with 512 maps 245 against 219 us)
    const double eff = c.shared ? std::min(0.88, 0.35 + 0.20 * wps) : std::min(0.95, 0.30 + 0.20 * wps);
    const double tail = wgs > res_wg ? rounds / (wgs / res_wg) : 1.0;
    // the shared-producer kernels run about 15 % faster than this count predicts (measured on the benchmark
    // shapes: fewer global loads per lane, no unpacking of x, step and mask in the scanning lanes)
    return wgs * c.waves * steps * 4.0 / (1024.0 * eff) * tail * (c.shared ? 0.85 : 1.0);
}

// sp: pick the instantiation that computes the step itself
// cf: columns first inside the kernel; only the shared-producer form has such instantiations (SCAN2D_ERR_BAD_SHAPE
//     when none of them takes the shape: the caller then runs columns first through transposes)
int choose_fwd(const scan2d_desc* d, FwdChoice* out, bool sp = false, bool ma = true, bool cf = false) {
    const TuneValues tsh = tune_get(kTuneShared);
    if (tsh.n >= 5 && fill_shared(d, tsh.v[0], tsh.v[1], tsh.v[2], tsh.v[3], tsh.v[4], sp, out, cf, tsh.n >= 6 && tsh.v[5] != 0 && !cf)) return SCAN2D_OK;
    if (cf) {
        bool any = false;
        double low = 0.0;
        for (const V6& v : kFwdSharedVariants) {
            FwdChoice c;
            if (v.NG * v.NW != d->N || !fill_shared(d, v.LG, v.K, v.NW, v.waves, v.RPB, sp, &c, true)) continue;
            const double cost = fwd_cost(d, c);
            if (!any || cost < low) { low = cost; *out = c; any = true; }
        }
        return any ? SCAN2D_OK : SCAN2D_ERR_BAD_SHAPE;
    }
    const TuneValues tf = tune_get(kTuneFwd);
    if (tf.n >= 2) {                                               // tuning aid: LG,K,NW,WAVES[,RPB]
        const int LG = tf.v[0], K = tf.v[1], NW = tf.v[2], waves = tf.n >= 4 ? tf.v[3] : 4, rpb = tf.n >= 5 ? tf.v[4] : 0;
        const int got = tf.n;
        if (got >= 2 && LG == 16 && (K == 1 || K == 2) && fill_small(d, K, sp, out)) return SCAN2D_OK;
        if (got >= 3 && (LG == 16 || LG == 32 || LG == 64) && NW >= 1 && (waves == 4 || waves == 8 || waves == 16) &&
            fill_choice(d, LG, K, NW, waves, rpb, sp, ma, out))
            return SCAN2D_OK;
    }
    // narrow maps: one column per lane up to 16 columns; two per lane up to 32 where the width rules out
    // the unguarded wide loads of the 4-column variants (measured: twice as fast as their guarded form)
    if (fill_tile16(d, sp, out)) return SCAN2D_OK;
    if (d->W <= 16 && fill_small(d, 1, sp, out)) return SCAN2D_OK;
    if (d->W <= 32 && d->W % 4 != 0 && fill_small(d, 2, sp, out)) return SCAN2D_OK;
    bool found = false;
    double best = 0.0;
    for (const V4& v : kFwdVariants) {
        FwdChoice c;
        if (!fill_choice(d, v.LG, v.K, v.NW, v.waves, 0, sp, ma, &c)) continue;
        const double cost = fwd_cost(d, c);
        if (!found || cost < best) { best = cost; *out = c; found = true; }
    }
    if (!(tsh.n == 1 && tsh.v[0] == 0))                              // override "0": never the shared-producer form
        for (const V6& v : kFwdSharedVariants) {
            FwdChoice c;
            if (v.NG * v.NW != d->N || !fill_shared(d, v.LG, v.K, v.NW, v.waves, v.RPB, sp, &c)) continue;
            const double cost = fwd_cost(d, c);
            if (!found || cost < best) { best = cost; *out = c; found = true; }
        }
    return found ? SCAN2D_OK : SCAN2D_ERR_BAD_SHAPE;
}

}  // namespace
// Kernels that use more than 64 KB of dynamic LDS need the attribute raised once per (device, kernel); the
// pairs already done are remembered so that a launch (possibly under stream capture) makes no attribute call.
bool allow_large_lds(const void* kernel, size_t bytes) {
    struct Done { int dev; const void* kernel; size_t bytes; };
    static std::mutex mu;
    static Done done[256];
    static int ndone = 0;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return false;
    std::lock_guard<std::mutex> lock(mu);
    for (int i = 0; i < ndone; ++i)
        if (done[i].dev == dev && done[i].kernel == kernel && done[i].bytes >= bytes) return true;
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    if (ndone < 256) done[ndone++] = Done{dev, kernel, bytes};
    return true;
}
namespace {

// Workspace of the scan kernel itself: row-end states between column panels (wide maps).
size_t fwd_workspace(const scan2d_desc* d, const FwdChoice& c) {
    if (!c.multi) return 0;
    return (size_t)d->Bt * d->Dc * d->N * d->H * sizeof(float);
}

}  // namespace
}  // namespace scan2d

using namespace scan2d;

namespace {
// ---- columns first: the same descriptor with H and W exchanged, and the transposed copies in the workspace
bool columns_first(const scan2d_desc* d) { return (d->flags & SCAN2D_FLAG_COLUMNS_FIRST) != 0; }
scan2d_desc swapped(const scan2d_desc* d) {
    scan2d_desc t = *d;
    t.H = d->W; t.W = d->H; t.flags = d->flags & ~(uint32_t)SCAN2D_FLAG_COLUMNS_FIRST;
    return t;
}
// Columns first inside the kernels (the same descriptor, no transposes): the forward when a shared-producer tiling
// takes the shape, the backward when its plan is the banded form with the shared-producer main sweep.  Everything
// else goes through the transposed copies.
bool fwd_fused_cf(const scan2d_desc* d) {
    FwdChoice ch;
    return columns_first(d) && choose_fwd(d, &ch, false, true, true) == SCAN2D_OK;
}
bool bwd_fused_cf(const scan2d_desc* d, bool softplus) { return columns_first(d) && bwd_workspace_bytes(d, softplus) != 0; }
scan2d_desc rows_first(const scan2d_desc* d) {
    scan2d_desc t = *d;
    t.flags = d->flags & ~(uint32_t)SCAN2D_FLAG_COLUMNS_FIRST;
    return t;
}
struct Regions {                                 // byte offsets behind the inner call's own workspace
    size_t x, delta, dy, dx, ddelta, Bm, Cm, dBm, dCm, mask, y, total;
};
Regions regions(const scan2d_desc* d, bool backward) {
    const size_t e = d->dtype == SCAN2D_BF16 ? 2 : 4, HW = (size_t)d->H * d->W;
    const size_t maps = align256((size_t)d->Bt * d->Dc * HW * e), st = align256((size_t)d->Bt * d->N * HW * e);
    const size_t stf = align256((size_t)d->Bt * d->N * HW * 4), mk = align256((size_t)d->Bt * HW);
    Regions r{};
    size_t o = 0;
    r.x = o; o += maps; r.delta = o; o += maps; r.Bm = o; o += st; r.Cm = o; o += st; r.mask = o; o += mk;
    if (backward) { r.dy = o; o += maps; r.dx = o; o += maps; r.ddelta = o; o += maps; r.dBm = o; o += stf; r.dCm = o; o += stf; }
    else { r.y = o; o += maps; }
    r.total = o;
    return r;
}

// Workspace of a forward call / of a backward call without the gate's own buffer; 0 = none, or no plan.
size_t fwd_need(const scan2d_desc* d) {
    if (fwd_fused_cf(d)) {
        const scan2d_desc t = rows_first(d);
        return fwd_need(&t);
    }
    if (columns_first(d)) {
        const scan2d_desc t = swapped(d);
        return align256(fwd_need(&t)) + regions(d, false).total;
    }
    // the variant may depend on whether the step is computed in the kernel and on the mask alignment (the cost
    // model knows their register counts): size the workspace for the largest of the four cases
    size_t inner = 0;
    for (int sp = 0; sp < 2; ++sp)
        for (int ma = 0; ma < 2; ++ma) {
            FwdChoice ch;
            if (choose_fwd(d, &ch, sp != 0, ma != 0) == SCAN2D_OK) inner = std::max(inner, fwd_workspace(d, ch));
        }
    const size_t sk = skip_bytes(d);
    return sk > 0 ? align256(inner) + sk : inner;
}
size_t bwd_need(const scan2d_desc* d, bool softplus) {
    if (columns_first(d) && !bwd_fused_cf(d, softplus)) {
        const scan2d_desc t = swapped(d);
        const size_t inner = bwd_need(&t, softplus);
        return inner == 0 ? 0 : align256(inner) + regions(d, true).total;
    }
    const size_t inner = bwd_workspace_bytes(d, softplus);
    return inner == 0 ? 0 : inner + skip_bytes(d);
}

// z, y_gated (softplus form only): where the chosen kernel has an instantiation with the output gate, it also writes
// y_gated = y * SiLU(z) (and y only if y != y_gated) and *gated is set; otherwise the call is the ungated one.
int fwd_impl(const scan2d_desc* desc, const void* x, const void* delta, const float* delta_bias, int softplus, const float* A,
             const void* Bm, const void* Cm, const float* Dskip, const uint8_t* mask,
             void* y, void* workspace, size_t workspace_bytes, void* stream,
             const void* z = nullptr, void* y_gated = nullptr, bool* gated = nullptr);

// Everything the scan launch of fwd_impl could refuse for this descriptor, without enqueuing anything.
int fwd_check(const scan2d_desc* d, bool sp, bool has_mask, bool cf) {
    FwdChoice ch;
    const int rc = choose_fwd(d, &ch, sp, !has_mask || (d->W % 4) == 0, cf);
    if (rc != SCAN2D_OK) return rc;
    const long long maps = (long long)d->Bt * d->Dc;
    if ((maps + ch.MPW - 1) / ch.MPW > 2147483647LL) return SCAN2D_ERR_BAD_SHAPE;
    const long long chunks = ((long long)d->H * d->W + 1023) / 1024;
    if (skip_bytes(d) > 0 && has_mask && chunks * maps > 2147483647LL) return SCAN2D_ERR_BAD_SHAPE;
    return SCAN2D_OK;
}

int fwd_columns_first(const scan2d_desc* desc, const void* x, const void* delta, const float* delta_bias, int softplus,
                      const float* A, const void* Bm, const void* Cm, const float* Dskip, const uint8_t* mask,
                      void* y, void* workspace, size_t workspace_bytes, void* stream) {
    const scan2d_desc t = swapped(desc);
    int rc = fwd_check(&t, softplus != 0, mask != nullptr, false);             // nothing is enqueued for a call that will fail
    if (rc != SCAN2D_OK) return rc;
    const size_t inner = align256(fwd_need(&t));
    const Regions r = regions(desc, false);
    if (workspace == nullptr || workspace_bytes < inner + r.total) return SCAN2D_ERR_WORKSPACE_SMALL;
    char* base = static_cast<char*>(workspace) + inner;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int e = desc->dtype == SCAN2D_BF16 ? 2 : 4;
    const long long maps = (long long)desc->Bt * desc->Dc, planes = (long long)desc->Bt * desc->N;
    rc = transpose_launch(e, x, base + r.x, maps, desc->H, desc->W, st);
    if (rc == SCAN2D_OK) rc = transpose_launch(e, delta, base + r.delta, maps, desc->H, desc->W, st);
    if (rc == SCAN2D_OK) rc = transpose_launch(e, Bm, base + r.Bm, planes, desc->H, desc->W, st);
    if (rc == SCAN2D_OK) rc = transpose_launch(e, Cm, base + r.Cm, planes, desc->H, desc->W, st);
    if (rc == SCAN2D_OK && mask != nullptr) rc = transpose_launch(1, mask, base + r.mask, desc->Bt, desc->H, desc->W, st);
    if (rc != SCAN2D_OK) return rc;
    rc = fwd_impl(&t, base + r.x, base + r.delta, delta_bias, softplus, A, base + r.Bm, base + r.Cm, Dskip,
                  mask != nullptr ? reinterpret_cast<const uint8_t*>(base + r.mask) : nullptr, base + r.y, workspace, inner, stream);
    if (rc != SCAN2D_OK) return rc;
    return transpose_launch(e, base + r.y, y, maps, t.H, t.W, st);
}

int fwd_impl(const scan2d_desc* desc, const void* x, const void* delta, const float* delta_bias, int softplus, const float* A,
             const void* Bm, const void* Cm, const float* Dskip, const uint8_t* mask,
             void* y, void* workspace, size_t workspace_bytes, void* stream, const void* z, void* y_gated, bool* gated) {
    int rc = check_desc(desc);
    if (rc != SCAN2D_OK) return rc;
    if (!x || !delta || !A || !Bm || !Cm || !y) return SCAN2D_ERR_NULL_POINTER;
    if (!aligned16(x) || !aligned16(delta) || !aligned16(A) || !aligned16(Bm) || !aligned16(Cm) ||
        !aligned16(y) || !aligned16(Dskip) || !aligned16(mask) || !aligned16(workspace) || !aligned16(delta_bias))
        return SCAN2D_ERR_MISALIGNED;
    rc = check_device();
    if (rc != SCAN2D_OK) return rc;
    const bool cf = fwd_fused_cf(desc);
    if (columns_first(desc) && !cf)
        return fwd_columns_first(desc, x, delta, delta_bias, softplus, A, Bm, Cm, Dskip, mask, y, workspace, workspace_bytes, stream);
    rc = fwd_check(desc, softplus != 0, mask != nullptr, cf);                  // nothing is enqueued for a call that will fail
    if (rc != SCAN2D_OK) return rc;
    FwdChoice ch;
    rc = choose_fwd(desc, &ch, softplus != 0, mask == nullptr || (desc->W % 4) == 0, cf);
    if (rc != SCAN2D_OK) return rc;
    const size_t sk = skip_bytes(desc);
    const size_t need = sk > 0 ? align256(fwd_workspace(desc, ch)) : fwd_workspace(desc, ch);
    if (need + sk > 0 && (workspace == nullptr || workspace_bytes < need + sk)) return SCAN2D_ERR_WORKSPACE_SMALL;
    if (sk > 0 && mask != nullptr) {       // identity cells: the kernels run on a copy of the step that is 0 under the mask
        void* step = static_cast<char*>(workspace) + need;
        rc = skip_step_launch(desc, delta, mask, softplus != 0, step, static_cast<hipStream_t>(stream));
        if (rc != SCAN2D_OK) return rc;
        delta = step;
    }

    FwdArgs a;
    a.x = x; a.delta = delta; a.A = A; a.Bm = Bm; a.Cm = Cm; a.Dskip = Dskip; a.mask = mask; a.y = y;
    a.delta_bias = delta_bias;
    a.carry = static_cast<float*>(workspace);
    a.maps = (long long)desc->Bt * desc->Dc;
    a.Dc = desc->Dc; a.H = desc->H; a.W = desc->W; a.N = desc->N;
    a.NG = ch.NG; a.MPW = ch.MPW; a.panels = ch.panels; a.RPB = ch.RPB;
    const long long wgs = (a.maps + ch.MPW - 1) / ch.MPW;
    if (wgs > 2147483647LL) return SCAN2D_ERR_BAD_SHAPE;
    if (z != nullptr && y_gated != nullptr && softplus != 0 && ch.shared && !ch.cf && !ch.skew) {   // the gate in the same kernel
        const bool ua = desc->dtype == SCAN2D_BF16 && (desc->W % 2) != 0;
        const FwdKernel k = desc->dtype == SCAN2D_BF16 ? fwd_shared_kernel_gate_bf16(ch.LG, ch.K, ch.NW, ch.NG, ch.waves, ch.RPB, ua)
                                                       : fwd_shared_kernel_gate_f32(ch.LG, ch.K, ch.NW, ch.NG, ch.waves, ch.RPB);
        if (k != nullptr) {
            ch.kernel = k;
            a.z = z; a.y_gated = y_gated;
            if (y == y_gated) a.y = nullptr;
            if (gated != nullptr) *gated = true;
        }
    }
    (void)hipGetLastError();
    if (ch.lds_bytes > 65536 && !allow_large_lds(reinterpret_cast<const void*>(ch.kernel), ch.lds_bytes)) return SCAN2D_ERR_LAUNCH_FAILED;
    hipLaunchKernelGGL(ch.kernel, dim3((unsigned)wgs), dim3(ch.waves * 64), ch.lds_bytes, static_cast<hipStream_t>(stream), a);
    return hipGetLastError() == hipSuccess ? SCAN2D_OK : SCAN2D_ERR_LAUNCH_FAILED;
}
}  // namespace

extern "C" int scan2d_fwd(const scan2d_desc* desc, const void* x, const void* delta, const float* A,
                          const void* Bm, const void* Cm, const float* Dskip, const uint8_t* mask,
                          void* y, void* workspace, size_t workspace_bytes, void* stream) {
    return fwd_impl(desc, x, delta, nullptr, 0, A, Bm, Cm, Dskip, mask, y, workspace, workspace_bytes, stream);
}

extern "C" int scan2d_fwd_softplus(const scan2d_desc* desc, const void* x, const void* delta_raw, const float* delta_bias,
                                   const float* A, const void* Bm, const void* Cm, const float* Dskip,
                                   const uint8_t* mask, void* y, void* workspace, size_t workspace_bytes, void* stream) {
    return fwd_impl(desc, x, delta_raw, delta_bias, 1, A, Bm, Cm, Dskip, mask, y, workspace, workspace_bytes, stream);
}

namespace {
// The backward of the scan proper: identity cells, sweeps, reductions.
int bwd_core(const scan2d_desc* desc, const void* x, const void* delta, const float* delta_bias, bool softplus,
             const float* A, const void* Bm, const void* Cm, const float* Dskip, const uint8_t* mask,
             const void* dy, void* dx, void* ddelta, float* ddelta_bias, float* dA, float* dBm, float* dCm,
             float* dDskip, void* workspace, size_t workspace_bytes, void* stream,
             const void* z = nullptr, const void* y_scan = nullptr, void* dz = nullptr) {
    int rc = bwd_check(desc, softplus);                                        // nothing is enqueued for a call that will fail
    if (rc != SCAN2D_OK) return rc;
    const size_t sk = skip_bytes(desc);
    if (sk > 0) {                // identity cells: the sweeps run on a copy of the step that is 0 under the mask
        const size_t inner = bwd_workspace_bytes(desc, softplus);
        if (inner == 0) return SCAN2D_ERR_BAD_SHAPE;
        if (workspace == nullptr || workspace_bytes < inner + sk) return SCAN2D_ERR_WORKSPACE_SMALL;
        if (mask != nullptr) {
            void* step = static_cast<char*>(workspace) + inner;
            rc = skip_step_launch(desc, delta, mask, softplus, step, static_cast<hipStream_t>(stream));
            if (rc != SCAN2D_OK) return rc;
            delta = step;
        }
        workspace_bytes = inner;
    }
    rc = bwd_launch(desc, x, delta, delta_bias, softplus, A, Bm, Cm, Dskip, mask, dy, dx, ddelta, ddelta_bias, dA, dBm, dCm,
                    dDskip, workspace, workspace_bytes, static_cast<hipStream_t>(stream), nullptr, nullptr, nullptr, z, y_scan, dz);
    // identity cells: their step is the constant 0, so it has no gradient (with the softplus step the chain
    // rule has already multiplied by the logistic function of -inf, which is 0)
    if (rc == SCAN2D_OK && sk > 0 && mask != nullptr && !softplus)
        rc = skip_grad_launch(desc, mask, ddelta, static_cast<hipStream_t>(stream));
    return rc;
}

int bwd_columns_first(const scan2d_desc* desc, const void* x, const void* delta, const float* delta_bias, bool softplus,
                      const float* A, const void* Bm, const void* Cm, const float* Dskip, const uint8_t* mask,
                      const void* dy, void* dx, void* ddelta, float* ddelta_bias, float* dA, float* dBm, float* dCm,
                      float* dDskip, void* workspace, size_t workspace_bytes, void* stream) {
    const scan2d_desc t = swapped(desc);
    int rc = bwd_check(&t, softplus);                                          // nothing is enqueued for a call that will fail
    if (rc != SCAN2D_OK) return rc;
    const size_t need = bwd_need(&t, softplus);
    if (need == 0) return SCAN2D_ERR_BAD_SHAPE;
    const size_t inner = align256(need);
    const Regions r = regions(desc, true);
    if (workspace == nullptr || workspace_bytes < inner + r.total) return SCAN2D_ERR_WORKSPACE_SMALL;
    char* base = static_cast<char*>(workspace) + inner;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int e = desc->dtype == SCAN2D_BF16 ? 2 : 4;
    const long long maps = (long long)desc->Bt * desc->Dc, planes = (long long)desc->Bt * desc->N;
    rc = transpose_launch(e, x, base + r.x, maps, desc->H, desc->W, st);
    if (rc == SCAN2D_OK) rc = transpose_launch(e, delta, base + r.delta, maps, desc->H, desc->W, st);
    if (rc == SCAN2D_OK) rc = transpose_launch(e, dy, base + r.dy, maps, desc->H, desc->W, st);
    if (rc == SCAN2D_OK) rc = transpose_launch(e, Bm, base + r.Bm, planes, desc->H, desc->W, st);
    if (rc == SCAN2D_OK) rc = transpose_launch(e, Cm, base + r.Cm, planes, desc->H, desc->W, st);
    if (rc == SCAN2D_OK && mask != nullptr) rc = transpose_launch(1, mask, base + r.mask, desc->Bt, desc->H, desc->W, st);
    if (rc != SCAN2D_OK) return rc;
    rc = bwd_core(&t, base + r.x, base + r.delta, delta_bias, softplus, A, base + r.Bm, base + r.Cm, Dskip,
                  mask != nullptr ? reinterpret_cast<const uint8_t*>(base + r.mask) : nullptr, base + r.dy, base + r.dx,
                  base + r.ddelta, ddelta_bias, dA, reinterpret_cast<float*>(base + r.dBm), reinterpret_cast<float*>(base + r.dCm),
                  dDskip, workspace, inner, stream);
    if (rc != SCAN2D_OK) return rc;
    rc = transpose_launch(e, base + r.dx, dx, maps, t.H, t.W, st);
    if (rc == SCAN2D_OK) rc = transpose_launch(e, base + r.ddelta, ddelta, maps, t.H, t.W, st);
    if (rc == SCAN2D_OK) rc = transpose_launch(4, base + r.dBm, dBm, planes, t.H, t.W, st);
    if (rc == SCAN2D_OK) rc = transpose_launch(4, base + r.dCm, dCm, planes, t.H, t.W, st);
    return rc;
}

int bwd_impl(const scan2d_desc* desc, const void* x, const void* delta, const float* delta_bias, bool softplus,
             const float* A, const void* Bm, const void* Cm, const float* Dskip, const uint8_t* mask,
             const void* dy, void* dx, void* ddelta, float* ddelta_bias, float* dA, float* dBm, float* dCm,
             float* dDskip, void* workspace, size_t workspace_bytes, void* stream,
             const void* z = nullptr, const void* y_scan = nullptr, void* dyg = nullptr, void* dz = nullptr) {
    int rc = check_desc(desc);
    if (rc != SCAN2D_OK) return rc;
    if (!x || !delta || !A || !Bm || !Cm || !dy || !dx || !ddelta || !dA || !dBm || !dCm)
        return SCAN2D_ERR_NULL_POINTER;
    if ((Dskip == nullptr) != (dDskip == nullptr)) return SCAN2D_ERR_NULL_POINTER;
    if ((delta_bias == nullptr) != (ddelta_bias == nullptr)) return SCAN2D_ERR_NULL_POINTER;
    const void* ptrs[] = {x, delta, A, Bm, Cm, Dskip, mask, dy, dx, ddelta, dA, dBm, dCm, dDskip, workspace, delta_bias, ddelta_bias};
    for (const void* q : ptrs)
        if (!aligned16(q)) return SCAN2D_ERR_MISALIGNED;
    rc = check_device();
    if (rc != SCAN2D_OK) return rc;
    // output gate: where the main sweep has an instantiation for it, dz and dy * SiLU(z) are formed where the sweep
    // produces its cells (nothing rounded in between); otherwise by an element-wise kernel in front of the sweeps
    const bool gate_in_sweep = z != nullptr && softplus && bwd_gate_in_sweep(desc);
    if (z != nullptr && !gate_in_sweep) {
        rc = gate_bwd_launch(desc, z, y_scan, dy, dyg, dz, static_cast<hipStream_t>(stream));
        if (rc != SCAN2D_OK) return rc;
        dy = dyg;
    }
    if (columns_first(desc) && !bwd_fused_cf(desc, softplus))
        return bwd_columns_first(desc, x, delta, delta_bias, softplus, A, Bm, Cm, Dskip, mask, dy, dx, ddelta, ddelta_bias, dA, dBm,
                                 dCm, dDskip, workspace, workspace_bytes, stream);
    return bwd_core(desc, x, delta, delta_bias, softplus, A, Bm, Cm, Dskip, mask, dy, dx, ddelta, ddelta_bias, dA, dBm, dCm,
                    dDskip, workspace, workspace_bytes, stream, gate_in_sweep ? z : nullptr, y_scan, dz);
}
}  // namespace

extern "C" int scan2d_bwd(const scan2d_desc* desc, const void* x, const void* delta, const float* A,
                          const void* Bm, const void* Cm, const float* Dskip, const uint8_t* mask,
                          const void* dy, void* dx, void* ddelta, float* dA, float* dBm, float* dCm,
                          float* dDskip, void* workspace, size_t workspace_bytes, void* stream) {
    return bwd_impl(desc, x, delta, nullptr, false, A, Bm, Cm, Dskip, mask, dy, dx, ddelta, nullptr, dA, dBm, dCm, dDskip,
                    workspace, workspace_bytes, stream);
}

extern "C" int scan2d_bwd_softplus(const scan2d_desc* desc, const void* x, const void* delta_raw, const float* delta_bias,
                                   const float* A, const void* Bm, const void* Cm, const float* Dskip, const uint8_t* mask,
                                   const void* dy, void* dx, void* ddelta_raw, float* ddelta_bias, float* dA, float* dBm,
                                   float* dCm, float* dDskip, void* workspace, size_t workspace_bytes, void* stream) {
    return bwd_impl(desc, x, delta_raw, delta_bias, true, A, Bm, Cm, Dskip, mask, dy, dx, ddelta_raw, ddelta_bias, dA, dBm, dCm,
                    dDskip, workspace, workspace_bytes, stream);
}

// Gated forward: the scan writes its output to y_scan (to y when the caller does not want y_scan), then one
// element-wise pass applies the gate.
extern "C" int scan2d_fwd_softplus_gated(const scan2d_desc* desc, const void* x, const void* delta_raw, const float* delta_bias,
                                         const float* A, const void* Bm, const void* Cm, const float* Dskip,
                                         const uint8_t* mask, const void* z, void* y_scan, void* y, void* workspace,
                                         size_t workspace_bytes, void* stream) {
    if (!z || !y) return SCAN2D_ERR_NULL_POINTER;
    if (!aligned16(z) || !aligned16(y_scan)) return SCAN2D_ERR_MISALIGNED;
    void* ys = y_scan != nullptr ? y_scan : y;
    bool gated = false;
    const int rc = fwd_impl(desc, x, delta_raw, delta_bias, 1, A, Bm, Cm, Dskip, mask, ys, workspace, workspace_bytes, stream, z, y, &gated);
    if (rc != SCAN2D_OK || gated) return rc;
    return gate_fwd_launch(desc, ys, z, y, static_cast<hipStream_t>(stream));
}

extern "C" int scan2d_bwd_softplus_gated(const scan2d_desc* desc, const void* x, const void* delta_raw, const float* delta_bias,
                                         const float* A, const void* Bm, const void* Cm, const float* Dskip, const uint8_t* mask,
                                         const void* z, const void* y_scan, const void* dy, void* dx, void* ddelta_raw,
                                         float* ddelta_bias, float* dA, float* dBm, float* dCm, float* dDskip, void* dz,
                                         void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_desc(desc);
    if (rc != SCAN2D_OK) return rc;
    if (!z || !y_scan || !dy || !dz) return SCAN2D_ERR_NULL_POINTER;
    if (!aligned16(z) || !aligned16(y_scan) || !aligned16(dy) || !aligned16(dz) || !aligned16(workspace)) return SCAN2D_ERR_MISALIGNED;
    const size_t inner = align256(bwd_need(desc, true));
    if (inner == 0) return SCAN2D_ERR_BAD_SHAPE;
    if (workspace == nullptr || workspace_bytes < inner + gate_bwd_bytes(desc)) return SCAN2D_ERR_WORKSPACE_SMALL;
    // the gate only changes dy: dy * SiLU(z) goes behind the scan's own workspace, dz is final
    void* dyg = static_cast<char*>(workspace) + inner;
    return bwd_impl(desc, x, delta_raw, delta_bias, true, A, Bm, Cm, Dskip, mask, dy, dx, ddelta_raw, ddelta_bias, dA, dBm, dCm,
                    dDskip, workspace, inner, stream, z, y_scan, dyg, dz);
}

namespace {
size_t variants_fwd_need(const scan2d_desc* d, bool av, bool pad);
size_t variants_bwd_need(const scan2d_desc* d, bool av, bool pad);
}  // namespace

extern "C" size_t scan2d_workspace_bytes(const scan2d_desc* desc, int pass) {
    if (check_desc(desc) != SCAN2D_OK) return 0;
    if (pass == SCAN2D_PASS_FWD) return fwd_need(desc);
    if (pass == SCAN2D_PASS_FWD_VARIANTS || pass == SCAN2D_PASS_BWD_VARIANTS) {   // enough for any combination of the variants
        if (desc->flags != 0u) return 0;
        size_t need = 0;
        for (int av = 0; av < 2; ++av)
            need = std::max(need, pass == SCAN2D_PASS_FWD_VARIANTS ? variants_fwd_need(desc, av != 0, true) : variants_bwd_need(desc, av != 0, true));
        return need;
    }
    if (pass == SCAN2D_PASS_BWD || pass == SCAN2D_PASS_BWD_SOFTPLUS || pass == SCAN2D_PASS_BWD_GATED) {
        const size_t inner = bwd_need(desc, pass != SCAN2D_PASS_BWD);
        if (inner == 0) return 0;
        return pass == SCAN2D_PASS_BWD_GATED ? align256(inner) + gate_bwd_bytes(desc) : inner;
    }
    return 0;
}

extern "C" int scan2d_describe_plan(const scan2d_desc* desc, int pass, char* text, size_t text_bytes) {
    if (text == nullptr || text_bytes == 0) return SCAN2D_ERR_NULL_POINTER;
    text[0] = 0;
    int rc = check_desc(desc);
    if (rc != SCAN2D_OK) return rc;
    const bool bwd_pass = pass == SCAN2D_PASS_BWD || pass == SCAN2D_PASS_BWD_SOFTPLUS || pass == SCAN2D_PASS_BWD_GATED;
    const bool fused = pass == SCAN2D_PASS_FWD ? fwd_fused_cf(desc) : (bwd_pass && bwd_fused_cf(desc, pass != SCAN2D_PASS_BWD));
    if (columns_first(desc) && !fused) {         // the plan of the kernels that run: those of the transposed maps
        const scan2d_desc t = swapped(desc);
        const int n = std::snprintf(text, text_bytes, "columns-first(transposed) ");
        if (n < 0 || (size_t)n >= text_bytes) return SCAN2D_OK;
        return scan2d_describe_plan(&t, pass, text + n, text_bytes - (size_t)n);
    }
    if (pass == SCAN2D_PASS_BWD_SOFTPLUS || pass == SCAN2D_PASS_BWD_GATED) pass = SCAN2D_PASS_BWD;   // the same sweeps
    if (pass == SCAN2D_PASS_FWD) {
        FwdChoice ch;
        rc = choose_fwd(desc, &ch, false, true, fused);
        if (rc != SCAN2D_OK) return rc;
        const long long maps = (long long)desc->Bt * desc->Dc;
        std::snprintf(text, text_bytes, "%sfwd form=%s LG=%d K=%d NW=%d waves=%d RPB=%d NG=%d MPW=%d panels=%d fast=%d exact=%d wgs=%lld lds=%zu workspace=%zu",
                      fused ? "columns-first(in-kernel) " : "", ch.tile ? "tile16" : (ch.K < 4 ? "small" : (ch.skew ? "skew" : (ch.shared ? "shared" : "general"))), ch.LG, ch.K, ch.NW, ch.waves, ch.RPB, ch.NG, ch.MPW, ch.panels,
                      (int)ch.fast, (int)ch.exact, (maps + ch.MPW - 1) / ch.MPW, ch.lds_bytes, fwd_workspace(desc, ch));
        return SCAN2D_OK;
    }
    if (pass == SCAN2D_PASS_BWD) return bwd_describe(desc, text, text_bytes) ? SCAN2D_OK : SCAN2D_ERR_BAD_SHAPE;
    return SCAN2D_ERR_BAD_FLAGS;
}

extern "C" const char* scan2d_strerror(int code) {
    switch (code) {
        case SCAN2D_OK: return "success";
        case SCAN2D_ERR_NULL_POINTER: return "a required pointer is NULL (or dDskip/Dskip do not match)";
        case SCAN2D_ERR_BAD_SHAPE: return "bad shape: every dimension must be >= 1, N <= 64, N*H*W < 2^27";
        case SCAN2D_ERR_BAD_DTYPE: return "dtype must be SCAN2D_F32 or SCAN2D_BF16";
        case SCAN2D_ERR_BAD_FLAGS: return "flags holds a bit other than SCAN2D_FLAG_IDENTITY_CELLS and SCAN2D_FLAG_COLUMNS_FIRST";
        case SCAN2D_ERR_WORKSPACE_SMALL: return "workspace is NULL or smaller than scan2d_workspace_bytes()";
        case SCAN2D_ERR_MISALIGNED: return "a base pointer is not 16-byte aligned";
        case SCAN2D_ERR_LAUNCH_FAILED: return "the HIP runtime refused a kernel launch";
        case SCAN2D_ERR_UNSUPPORTED_DEVICE: return "the current device is not gfx950 (MI355X)";
        case SCAN2D_ERR_SCRATCH_LIMIT: return "scan2d_bwd_static_scratch: the call needs more workspace than the built-in scratch array holds (SCAN2D_STATIC_SCRATCH_BYTES); use scan2d_bwd with a workspace";
        default: return "unknown scan2d error code";
    }
}

// ------------------------------------------------------------------ the ablated variants: padding token, own vertical decay
namespace {
// Forward plan of the instantiation with an independent vertical decay: 16-lane groups of 4 columns and 4 states,
// guarded accesses, column panels - one kernel per storage type that covers every shape.
bool fill_av(const scan2d_desc* d, FwdChoice* out) {
    FwdChoice c;
    c.LG = 16; c.K = 4; c.NW = 4; c.waves = 4;
    c.exact = false; c.fast = false; c.multi = true;
    c.NG = (d->N + 3) / 4;
    const int slots = 16;
    if (c.NG > slots) return false;
    c.MPW = slots / c.NG;
    c.panels = (d->W + 63) / 64;
    const double span = (double)(slots + 1) * d->N * d->H * d->W * 4.0;
    if (span >= 2147483648.0) return false;
    c.kernel = d->dtype == SCAN2D_BF16 ? fwd_kernel_av_bf16() : fwd_kernel_av_f32();
    c.RPB = c.NG > 1 ? 2 : 1;
    c.lds_bytes = c.NG > 1 ? 2 * (size_t)c.RPB * 256 * 4 * sizeof(float) : 0;
    *out = c;
    return true;
}
size_t av_carry_bytes(const scan2d_desc* d, const FwdChoice& c) {
    return c.panels > 1 ? align256((size_t)d->Bt * d->Dc * d->N * d->H * sizeof(float)) : 0;
}
size_t map_bytes(const scan2d_desc* d) {
    return align256((size_t)d->Bt * d->Dc * d->H * d->W * (d->dtype == SCAN2D_BF16 ? 2 : 4));
}
// Workspace of the variant calls: [scan kernels][copy of x with the padding token][per-map sums of dpad]
size_t variants_fwd_need(const scan2d_desc* d, bool av, bool pad) {
    size_t inner;
    if (av) {
        FwdChoice c;
        if (!fill_av(d, &c)) return 0;
        inner = av_carry_bytes(d, c);
    } else {
        inner = align256(fwd_need(d));
    }
    return inner + (pad ? map_bytes(d) : 0);
}
size_t variants_bwd_need(const scan2d_desc* d, bool av, bool pad) {
    const size_t inner = bwd_workspace_bytes(d, false, av);
    if (inner == 0) return 0;
    return align256(inner) + (pad ? map_bytes(d) + align256((size_t)d->Bt * d->Dc * sizeof(float)) : 0);
}
}  // namespace

extern "C" int scan2d_fwd_variants(const scan2d_desc* desc, const void* x, const void* delta, const float* A,
                                   const void* Bm, const void* Cm, const float* Dskip, const uint8_t* mask,
                                   const scan2d_variants* v, void* y, void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_desc(desc);
    if (rc != SCAN2D_OK) return rc;
    if (desc->flags != 0u) return SCAN2D_ERR_BAD_FLAGS;
    if (!x || !delta || !A || !Bm || !Cm || !y) return SCAN2D_ERR_NULL_POINTER;
    const float* A_v = v != nullptr ? v->A_v : nullptr;
    const float* pad = (v != nullptr && mask != nullptr) ? v->pad : nullptr;      // without a mask the token is nowhere
    const void* ptrs[] = {x, delta, A, Bm, Cm, Dskip, mask, y, workspace, A_v, pad};
    for (const void* q : ptrs)
        if (!aligned16(q)) return SCAN2D_ERR_MISALIGNED;
    rc = check_device();
    if (rc != SCAN2D_OK) return rc;
    const size_t need = variants_fwd_need(desc, A_v != nullptr, pad != nullptr);
    if (need > 0 && (workspace == nullptr || workspace_bytes < need)) return SCAN2D_ERR_WORKSPACE_SMALL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const size_t inner = need - (pad != nullptr ? map_bytes(desc) : 0);
    if (pad != nullptr) {                      // the scan runs without a mask on a copy of x that holds the token
        void* xe = static_cast<char*>(workspace) + inner;
        rc = pad_fill_launch(desc, x, mask, pad, xe, st);
        if (rc != SCAN2D_OK) return rc;
        x = xe; mask = nullptr;
    }
    if (A_v == nullptr) return fwd_impl(desc, x, delta, nullptr, 0, A, Bm, Cm, Dskip, mask, y, workspace, inner, stream);
    FwdChoice ch;
    if (!fill_av(desc, &ch)) return SCAN2D_ERR_BAD_SHAPE;
    FwdArgs a;
    a.x = x; a.delta = delta; a.A = A; a.Bm = Bm; a.Cm = Cm; a.Dskip = Dskip; a.mask = mask; a.y = y;
    a.delta_bias = nullptr; a.A_v = A_v;
    a.carry = static_cast<float*>(workspace);
    a.maps = (long long)desc->Bt * desc->Dc;
    a.Dc = desc->Dc; a.H = desc->H; a.W = desc->W; a.N = desc->N;
    a.NG = ch.NG; a.MPW = ch.MPW; a.panels = ch.panels; a.RPB = ch.RPB;
    const long long wgs = (a.maps + ch.MPW - 1) / ch.MPW;
    if (wgs > 2147483647LL) return SCAN2D_ERR_BAD_SHAPE;
    (void)hipGetLastError();
    hipLaunchKernelGGL(ch.kernel, dim3((unsigned)wgs), dim3(ch.waves * 64), ch.lds_bytes, st, a);
    return hipGetLastError() == hipSuccess ? SCAN2D_OK : SCAN2D_ERR_LAUNCH_FAILED;
}

extern "C" int scan2d_bwd_variants(const scan2d_desc* desc, const void* x, const void* delta, const float* A,
                                   const void* Bm, const void* Cm, const float* Dskip, const uint8_t* mask,
                                   const scan2d_variants* v, const void* dy, void* dx, void* ddelta, float* dA, float* dBm,
                                   float* dCm, float* dDskip, void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_desc(desc);
    if (rc != SCAN2D_OK) return rc;
    if (desc->flags != 0u) return SCAN2D_ERR_BAD_FLAGS;
    if (!x || !delta || !A || !Bm || !Cm || !dy || !dx || !ddelta || !dA || !dBm || !dCm) return SCAN2D_ERR_NULL_POINTER;
    if ((Dskip == nullptr) != (dDskip == nullptr)) return SCAN2D_ERR_NULL_POINTER;
    const float* A_v = v != nullptr ? v->A_v : nullptr;
    float* dA_v = v != nullptr ? v->dA_v : nullptr;
    const float* pad = v != nullptr ? v->pad : nullptr;
    float* dpad = v != nullptr ? v->dpad : nullptr;
    if ((A_v == nullptr) != (dA_v == nullptr) || (pad == nullptr) != (dpad == nullptr)) return SCAN2D_ERR_NULL_POINTER;
    const void* ptrs[] = {x, delta, A, Bm, Cm, Dskip, mask, dy, dx, ddelta, dA, dBm, dCm, dDskip, workspace, A_v, dA_v, pad, dpad};
    for (const void* q : ptrs)
        if (!aligned16(q)) return SCAN2D_ERR_MISALIGNED;
    rc = check_device();
    if (rc != SCAN2D_OK) return rc;
    const size_t need = variants_bwd_need(desc, A_v != nullptr, pad != nullptr);
    if (need == 0) return SCAN2D_ERR_BAD_SHAPE;
    if (workspace == nullptr || workspace_bytes < need) return SCAN2D_ERR_WORKSPACE_SMALL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const size_t inner = align256(bwd_workspace_bytes(desc, false, A_v != nullptr));
    const uint8_t* scan_mask = mask;
    float* ppad = nullptr;
    if (pad != nullptr) {
        ppad = reinterpret_cast<float*>(static_cast<char*>(workspace) + inner + map_bytes(desc));
        if (mask != nullptr) {                 // the sweeps run without a mask on a copy of x that holds the token
            void* xe = static_cast<char*>(workspace) + inner;
            rc = pad_fill_launch(desc, x, mask, pad, xe, st);
            if (rc != SCAN2D_OK) return rc;
            x = xe; scan_mask = nullptr;
        }
    }
    rc = bwd_launch(desc, x, delta, nullptr, false, A, Bm, Cm, Dskip, scan_mask, dy, dx, ddelta, nullptr, dA, dBm, dCm, dDskip,
                    workspace, inner, st, A_v, dA_v);
    if (rc != SCAN2D_OK) return rc;
    // dx now holds the gradient of the copy: its sum over the masked cells is dpad, and dx itself is +0 there
    if (pad != nullptr) rc = pad_grad_launch(desc, mask, dx, ppad, dpad, st);
    return rc;
}

// ------------------------------------------------------------------ backward without a caller's workspace
// The workspace of this entry point: device memory that lives in the library's code object, one copy per GPU,
// from the moment the library is loaded on that GPU until the process ends.
static __device__ __align__(256) unsigned char scratch[SCAN2D_STATIC_SCRATCH_BYTES];

namespace {
std::atomic<void*> g_scratch_ptr[kMaxDevices];   // device address of `scratch` on each GPU, asked for once per device

// The array's name is a host-side handle, not a device address: kernels and copies get the address that the
// runtime reports for the current device.
void* scratch_address() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (p != nullptr) return p;
    void* q = nullptr;
    if (hipGetSymbolAddress(&q, HIP_SYMBOL(scratch)) != hipSuccess || q == nullptr) {
        (void)hipGetLastError();
        return nullptr;
    }
    g_scratch_ptr[dev].store(q, std::memory_order_release);
    return q;
}
}  // namespace

extern "C" int scan2d_bwd_static_scratch(const scan2d_desc* desc, const void* x, const void* delta, const float* A,
                                         const void* Bm, const void* Cm, const float* Dskip, const uint8_t* mask,
                                         const void* dy, void* dx, void* ddelta, float* dA, float* dBm, float* dCm,
                                         float* dDskip, void* stream) {
    int rc = check_desc(desc);
    if (rc != SCAN2D_OK) return rc;
    const size_t need = bwd_need(desc, false);
    if (need == 0) return SCAN2D_ERR_BAD_SHAPE;
    if (need > (size_t)SCAN2D_STATIC_SCRATCH_BYTES) return SCAN2D_ERR_SCRATCH_LIMIT;
    rc = check_device();
    if (rc != SCAN2D_OK) return rc;
    void* ws = scratch_address();
    if (ws == nullptr) return SCAN2D_ERR_LAUNCH_FAILED;
    return bwd_impl(desc, x, delta, nullptr, false, A, Bm, Cm, Dskip, mask, dy, dx, ddelta, nullptr, dA, dBm, dCm, dDskip,
                    ws, need, stream);
}

extern "C" size_t scan2d_saved_bytes(const scan2d_desc* desc) {
    if (check_desc(desc) != SCAN2D_OK || desc->flags != 0u) return 0;
    return bwd_saved_bytes(desc);
}

extern "C" int scan2d_fwd_saving(const scan2d_desc* desc, const void* x, const void* delta, const float* A, const void* Bm,
                                 const void* Cm, const float* Dskip, const uint8_t* mask, void* y, void* saved, size_t saved_bytes,
                                 void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_desc(desc);
    if (rc != SCAN2D_OK) return rc;
    if (desc->flags != 0u) return SCAN2D_ERR_BAD_FLAGS;
    const size_t need = bwd_saved_bytes(desc);
    if (need == 0) return fwd_impl(desc, x, delta, nullptr, 0, A, Bm, Cm, Dskip, mask, y, workspace, workspace_bytes, stream);
    if (!x || !delta || !A || !Bm || !Cm || !y || !saved) return SCAN2D_ERR_NULL_POINTER;
    if (!aligned16(x) || !aligned16(delta) || !aligned16(A) || !aligned16(Bm) || !aligned16(Cm) || !aligned16(y) ||
        !aligned16(Dskip) || !aligned16(mask) || !aligned16(saved))
        return SCAN2D_ERR_MISALIGNED;
    if (saved_bytes < need) return SCAN2D_ERR_WORKSPACE_SMALL;
    rc = check_device();
    if (rc != SCAN2D_OK) return rc;
    return fwd_saving_launch(desc, x, delta, A, Bm, Cm, Dskip, mask, y, static_cast<float*>(saved), static_cast<hipStream_t>(stream));
}

extern "C" int scan2d_bwd_saved(const scan2d_desc* desc, const void* x, const void* delta, const float* A, const void* Bm,
                                const void* Cm, const float* Dskip, const uint8_t* mask, const void* dy, const void* saved,
                                size_t saved_bytes, void* dx, void* ddelta, float* dA, float* dBm, float* dCm, float* dDskip,
                                void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_desc(desc);
    if (rc != SCAN2D_OK) return rc;
    if (desc->flags != 0u) return SCAN2D_ERR_BAD_FLAGS;
    const size_t need = bwd_saved_bytes(desc);
    if (need == 0)
        return bwd_impl(desc, x, delta, nullptr, false, A, Bm, Cm, Dskip, mask, dy, dx, ddelta, nullptr, dA, dBm, dCm, dDskip, workspace,
                        workspace_bytes, stream);
    if (!x || !delta || !A || !Bm || !Cm || !dy || !dx || !ddelta || !dA || !dBm || !dCm || !saved) return SCAN2D_ERR_NULL_POINTER;
    if ((Dskip == nullptr) != (dDskip == nullptr)) return SCAN2D_ERR_NULL_POINTER;
    const void* ptrs[] = {x, delta, A, Bm, Cm, Dskip, mask, dy, dx, ddelta, dA, dBm, dCm, dDskip, workspace, saved};
    for (const void* q : ptrs)
        if (!aligned16(q)) return SCAN2D_ERR_MISALIGNED;
    if (saved_bytes < need) return SCAN2D_ERR_WORKSPACE_SMALL;
    rc = check_device();
    if (rc != SCAN2D_OK) return rc;
    rc = bwd_check(desc, false);
    if (rc != SCAN2D_OK) return rc;
    return bwd_launch(desc, x, delta, nullptr, false, A, Bm, Cm, Dskip, mask, dy, dx, ddelta, nullptr, dA, dBm, dCm, dDskip, workspace,
                      workspace_bytes, static_cast<hipStream_t>(stream), nullptr, nullptr, static_cast<const float*>(saved));
}

extern "C" int scan2d_block_conv_silu(const scan2d_desc* desc, const scan2d_conv_shape* shape, const void* u, const float* w,
                                      const float* bias, void* x, void* stream) {
    int rc = check_desc(desc);
    if (rc != SCAN2D_OK) return rc;
    if (!shape || !u || !w || !x) return SCAN2D_ERR_NULL_POINTER;
    if (!aligned16(u) || !aligned16(w) || !aligned16(bias) || !aligned16(x)) return SCAN2D_ERR_MISALIGNED;
    if (u == x) return SCAN2D_ERR_BAD_SHAPE;                       // every output reads its neighbours' inputs
    rc = check_device();
    if (rc != SCAN2D_OK) return rc;
    return block_conv_silu_launch(desc, shape, u, w, bias, x, static_cast<hipStream_t>(stream));
}

extern "C" int scan2d_block_xproj(const scan2d_desc* desc, int R, const void* x, const void* Wx, const float* Wdt,
                                  void* delta_raw, void* Bm, void* Cm, void* stream) {
    int rc = check_desc(desc);
    if (rc != SCAN2D_OK) return rc;
    if (!x || !Wx || !Wdt || !delta_raw || !Bm || !Cm) return SCAN2D_ERR_NULL_POINTER;
    if (!aligned16(x) || !aligned16(Wx) || !aligned16(Wdt) || !aligned16(delta_raw) || !aligned16(Bm) || !aligned16(Cm))
        return SCAN2D_ERR_MISALIGNED;
    rc = check_device();
    if (rc != SCAN2D_OK) return rc;
    return block_xproj_launch(desc, R, x, Wx, Wdt, delta_raw, Bm, Cm, static_cast<hipStream_t>(stream));
}

extern "C" int scan2d_block_attn_pool(const scan2d_desc* desc, int D, const void* h, const void* V, const float* w,
                                      const uint8_t* mask, float* attn, float* z, void* stream) {
    int rc = check_desc(desc);
    if (rc != SCAN2D_OK) return rc;
    if (!h || !V || !w || !attn || !z) return SCAN2D_ERR_NULL_POINTER;
    if (!aligned16(h) || !aligned16(V) || !aligned16(w) || !aligned16(attn) || !aligned16(z) || (mask && !aligned16(mask)))
        return SCAN2D_ERR_MISALIGNED;
    rc = check_device();
    if (rc != SCAN2D_OK) return rc;
    return block_attn_pool_launch(desc, D, h, V, w, mask, attn, z, static_cast<hipStream_t>(stream));
}

extern "C" int scan2d_block_linear(const scan2d_desc* desc, int Cout, const void* in, const void* Wt, const float* bias,
                                   const void* residual, void* out, void* stream) {
    int rc = check_desc(desc);
    if (rc != SCAN2D_OK) return rc;
    if (!in || !Wt || !out) return SCAN2D_ERR_NULL_POINTER;
    if (!aligned16(in) || !aligned16(Wt) || !aligned16(out) || (bias && !aligned16(bias)) || (residual && !aligned16(residual)))
        return SCAN2D_ERR_MISALIGNED;
    if (in == out) return SCAN2D_ERR_BAD_SHAPE;           // every output reads all input channels of its position
    rc = check_device();
    if (rc != SCAN2D_OK) return rc;
    return block_linear_launch(desc, Cout, in, Wt, bias, residual, out, static_cast<hipStream_t>(stream));
}

extern "C" int scan2d_block_norm(const scan2d_desc* desc, int kind, float eps, const void* in, const float* gamma,
                                 const float* beta, void* out, void* stream) {
    int rc = check_desc(desc);
    if (rc != SCAN2D_OK) return rc;
    if (!in || !gamma || !out) return SCAN2D_ERR_NULL_POINTER;
    if (!aligned16(in) || !aligned16(gamma) || !aligned16(out) || (beta && !aligned16(beta))) return SCAN2D_ERR_MISALIGNED;
    rc = check_device();
    if (rc != SCAN2D_OK) return rc;
    return block_norm_launch(desc, kind, eps, in, gamma, beta, out, static_cast<hipStream_t>(stream));
}

extern "C" int scan2d_debug_force_variant(int kind, const int* values, int n) {
    if (kind < 0 || kind >= kTuneKinds) return SCAN2D_ERR_BAD_FLAGS;
    if (n > 0 && values == nullptr) return SCAN2D_ERR_NULL_POINTER;
    tune_set(kind, values, n);
    return SCAN2D_OK;
}

extern "C" int scan2d_version(void) { return 200; }
