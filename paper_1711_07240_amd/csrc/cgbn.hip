// Host side of libcgbn: argument validation, launch plan, launches, C ABI.
// See include/cgbn.h for the contract of every entry point.

#include "cgbn.h"
#include "cgbn_kernels.h"
#include "cgbn_fused.h"
#include "cgbn_fused_list.h"

#include <atomic>
#include <cmath>
#include <cstring>
#include <map>
#include <mutex>
#include <type_traits>
#include <utility>

// The NCHW single-launch kernels are instantiated in cgbn_fused_inst.hip (one translation
// unit per element type, direction and activation); here they are only declared.
namespace cgbn {
#define CGBN_DECL_FX(LB_, LPPC_, BIG_)                                                              \
    extern template __global__ void nchw_fused_forward<float, LB_, LPPC_, 0, BIG_>(FusedArgs);     \
    extern template __global__ void nchw_fused_forward<float, LB_, LPPC_, 1, BIG_>(FusedArgs);     \
    extern template __global__ void nchw_fused_forward<float, LB_, LPPC_, 2, BIG_>(FusedArgs);     \
    extern template __global__ void nchw_fused_forward<bf16_t, LB_, LPPC_, 2, BIG_>(FusedArgs);    \
    extern template __global__ void nchw_fused_forward<bf16_t, LB_, LPPC_, 0, BIG_>(FusedArgs);    \
    extern template __global__ void nchw_fused_forward<bf16_t, LB_, LPPC_, 1, BIG_>(FusedArgs);
#define CGBN_DECL_BX(LB_, LPPC_, BIG_)                                                              \
    extern template __global__ void nchw_fused_backward<float, LB_, LPPC_, 0, BIG_>(FusedArgs);    \
    extern template __global__ void nchw_fused_backward<float, LB_, LPPC_, 1, BIG_>(FusedArgs);    \
    extern template __global__ void nchw_fused_backward<bf16_t, LB_, LPPC_, 0, BIG_>(FusedArgs);   \
    extern template __global__ void nchw_fused_backward<bf16_t, LB_, LPPC_, 1, BIG_>(FusedArgs);
#define CGBN_DECL_F(LB_, LPPC_) CGBN_DECL_FX(LB_, LPPC_, 0)
#define CGBN_DECL_B(LB_, LPPC_) CGBN_DECL_BX(LB_, LPPC_, 0)
CGBN_FUSED_COMMON(CGBN_DECL_F)
CGBN_FUSED_FORWARD_ONLY(CGBN_DECL_F)
CGBN_FUSED_COMMON(CGBN_DECL_B)
CGBN_FUSED_BACKWARD_ONLY(CGBN_DECL_B)
CGBN_DECL_FX(16, 0, 1)
CGBN_DECL_BX(16, 0, 1)
CGBN_DECL_FX(16, -2, 1)
CGBN_DECL_BX(16, -2, 1)
#define CGBN_DECL_F1(LB_, LPPC_) CGBN_DECL_FX(LB_, LPPC_, 1)
#define CGBN_DECL_B1(LB_, LPPC_) CGBN_DECL_BX(LB_, LPPC_, 1)
CGBN_FUSED_WGP_FORWARD(CGBN_DECL_F1)
CGBN_FUSED_WGP_BACKWARD(CGBN_DECL_B1)
#undef CGBN_DECL_F1
#undef CGBN_DECL_B1
#define CGBN_DECL_F2(LB_, LPPC_) CGBN_DECL_FX(LB_, LPPC_, 2)
#define CGBN_DECL_B2(LB_, LPPC_) CGBN_DECL_BX(LB_, LPPC_, 2)
CGBN_FUSED_BIG_SMALL(CGBN_DECL_F2)
CGBN_FUSED_BIG_SMALL(CGBN_DECL_B2)
#undef CGBN_DECL_F2
#undef CGBN_DECL_B2
#undef CGBN_DECL_FX
#undef CGBN_DECL_BX
#undef CGBN_DECL_F
#undef CGBN_DECL_B
}  // namespace cgbn

// Scratch of cgbn_forward_static: one array per device, owned by the loaded library until the process ends.
// In host code this name is only a handle for hipGetSymbolAddress; kernels get the address that call returns.
static __device__ __align__(256) unsigned char scratch[CGBN_STATIC_SCRATCH_BYTES];

namespace {

using namespace cgbn;

// The device address of `scratch` on the current device, looked up once per device.
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices];
std::mutex g_scratch_lock;
cgbn_status scratch_of_current_device(void** out)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        return CGBN_ERR_HIP;
    }
    std::lock_guard<std::mutex> hold(g_scratch_lock);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
            (void)hipGetLastError();
            return CGBN_ERR_HIP;
        }
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return CGBN_OK;
}

// ---- launch-shape knobs (cgbn_set_tuning) ---------------------------------
struct Tuning {
    long long chunk_bytes = 32768;       // NCHW: bytes of a plane per workgroup
    long long wave_plane_bytes = 16384;  // NCHW: planes up to this go one per wavefront
    long long tiny_planes = 1;           // NCHW: planes of at most 2 KiB (C a multiple of 8) go several to a workgroup
    long long piece_bytes = 0;           // NHWC reductions: bytes of a pixel run per workgroup; 0 = chosen per shape (see reduce_pieces)
    long long map_piece_bytes = 0;       // NHWC normalise / dx: the same for the elementwise sweeps; 0 = chosen per dtype and sweep (see map_pieces)
    long long reverse = 1;               // alternate sweep direction so a sweep starts on what the last one left in cache
    long long nt_store = 1;              // non-temporal stores for y and dx
    long long fused = 1;                 // register-resident single-launch path where the shape allows it
    long long spin_limit = 1LL << 24;    // polls of a bounded wait in the fused kernels before it gives up
    long long cooperative = 0;           // launch the single-launch kernels cooperatively (co-residency guaranteed by the runtime)
    long long big_lds = 1;               // large planes with few rows/shards: keep more unit data in LDS
    long long one_sweep_stats = 1;       // multi-sweep forward: steps 1-10 from one sweep over x (0: a sweep for the sums, one for the deviations)
    long long fused_groups = 0;          // workgroups of the fused grid (0 = as many as are resident at once)
    long long stagger = 1;               // single-launch kernels: start the channel slots class by class (see choose_stagger)
    long long stagger_us = 0;            // ... start-up delay of the last class (0 = chosen per launch)
    long long stagger_phases = 16;       // ... and the number of classes
    long long wait_us = 100000;          // microseconds after which a device-side wait of the fused kernels gives up
};
// The knobs are process-wide; every call works on ONE copy of them taken under the lock when it starts
// (tuning_now), so a knob changed by another thread in the middle of a call cannot make the plan, the
// workspace check and the launches of that call disagree.
Tuning g_tune;
std::mutex g_tune_lock;
Tuning tuning_now()
{
    std::lock_guard<std::mutex> hold(g_tune_lock);
    return g_tune;
}
std::atomic<long long> g_last_forward_fused{0}, g_last_backward_fused{0};   // which path the last call took
#ifdef CGBN_TRACE
unsigned long long* g_trace = nullptr;
#endif

// Geometry of the register-resident path for one direction (`words` 32-bit
// registers of one tensor per thread: 128 forward, 64 backward).
struct FusedPlan {
    int ok;               // shape can take the path at all (grid size is checked at launch)
    int LB;               // bytes per load: 16 or 8
    int LPPC;             // 0: large planes; else register slots per plane (an instantiated count >= LPP)
    int tp, TL, LPP, IPU, U, rows, rps, G;
    int big;              // 1 (large planes) / 2 (small planes): the variant that stages few rows and keeps more unit data in LDS
    long long total_units;
};

struct Plan {
    Tuning t;             // the knobs this plan was made under (the call's own copy)
    int N, C, H, W, K, layout, dtype;
    int eb, vec;          // bytes per element; elements per 16-byte vector (NHWC: 1 if C is not a multiple)
    int HW, ips;
    long long S;
    double M;
    // NCHW
    int wave_mode, L, sp;
    int tiny, tg;         // tiny planes: `tg` planes of consecutive channels per workgroup
    // NHWC
    int cv, TW, ctiles, rpp, PL, pps;
    int PLm, ppsm;        // pixel runs of the elementwise sweeps (no rows to keep few): one input tensor ...
    int PLm2, ppsm2;      // ... and two or three (dx; the shortcut and ReLU variants)
    long long spix, gridm, gridm2;
    // partial sums
    int rows, rps, G;
    long long grid;       // workgroups of one sweep
    FusedPlan ff, fb;     // register-resident path, forward and backward
    // workspace layout (byte offsets)
    size_t off_part0, off_part1, off_sh0, off_sh1, off_mlo, off_sync, bytes;
};

size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

void make_fused_plan(const Tuning& T, int N, int C, long long HW, int K, int layout, int eb, int words, int lds_words,
                     int lds_words_big, int lds_words_big_small, bool forward, FusedPlan* f)
{
    std::memset(f, 0, sizeof(*f));
    if (K > kFusedMaxShards) return;
    if (layout != CGBN_NCHW) return;                   // channels-last shapes take the multi-sweep kernels
    int LB = 0;
    for (int lb = 16; lb >= 4; lb >>= 1)
        if (HW % (lb / eb) == 0) { LB = lb; break; }
    if (!LB) return;                                   // bfloat16 planes with an odd element count
    const int W = LB / 4, R = words / W, E = LB / eb;
    const long long wave_cap = (long long)R * kWave * E;   // elements one wavefront can hold
    if (LB == 4 && HW > wave_cap) return;              // 4-byte loads only for small planes
    const int ips = N / K;
    f->LB = LB;
    if (HW <= wave_cap) {
        f->LPP = (int)((HW + (long long)kWave * E - 1) / ((long long)kWave * E));
        // register slots per plane: the smallest instantiated count that holds a plane and
        // leaves at most 16 planes per wavefront
        int lppc = 0;
        for (int cand : kCgbnSlotCounts)
            if (cand >= f->LPP && cand * 16 >= R && cand <= R) { lppc = cand; break; }
        if (!lppc) return;
        if (f->LPP <= cgbn_full_slots(lppc, R)) return;    // (cannot happen: the kernels rely on it, see the table)
        f->LPPC = lppc;
        // with few rows and shards to stage, further whole planes per wavefront go to LDS
        int lds_planes = 0;
        if (T.big_lds && N <= kFusedMaxRowsBig && K <= kFusedMaxShardsBigSmall) {
            bool built = false;
#define CGBN_IS_BUILT(LB_, LPPC_) built = built || (LB == LB_ && lppc == LPPC_);
            CGBN_FUSED_BIG_SMALL(CGBN_IS_BUILT)
#undef CGBN_IS_BUILT
            if (built) lds_planes = (lds_words_big_small / W) / lppc;
            // ... if that makes the channel's units fewer (else the variant only costs its extra slot checks)
            const int regs_only = 4 * (R / lppc), with_lds = 4 * (R / lppc + lds_planes);
            if ((N + with_lds - 1) / with_lds >= (N + regs_only - 1) / regs_only) lds_planes = 0;
        }
        f->big = lds_planes > 0 ? 2 : 0;
        int per_unit = 4 * (R / lppc + lds_planes);
        f->U = (N + per_unit - 1) / per_unit;
        f->IPU = (N + f->U - 1) / f->U;
        // byte offsets inside a unit are 32-bit
        if ((long long)f->IPU * C * HW * eb > 0x7fffffffLL) return;
        f->rows = N;
        f->rps = ips;
    } else if (LB >= 8 && HW <= (long long)(R + lds_words / W) * kWave * E) {
        // a plane a few slots too long for a wavefront's registers: still one plane per wavefront, the last
        // slots in LDS (four planes per unit instead of the one a "large plane" unit would hold)
        f->LPP = (int)((HW + (long long)kWave * E - 1) / ((long long)kWave * E));
        f->LPPC = R + lds_words / W;
        f->U = (N + 3) / 4;
        f->IPU = (N + f->U - 1) / f->U;
        if ((long long)f->IPU * C * HW * eb > 0x7fffffffLL) return;
        f->rows = N;
        f->rps = ips;
    } else {
        // large planes: a tile also fills the LDS slots (16-byte loads only); with few rows and shards to
        // stage, the variant with more LDS slots is taken
        const long long gran = (long long)kThreads * E;
        for (int big = (LB == 16 && T.big_lds && K <= kFusedMaxShardsBig) ? 1 : 0; big >= 0; --big) {
            const int lw = big ? lds_words_big : lds_words;
            const long long cap = wave_cap * 4 + (LB == 16 ? (long long)(lw / W) * kThreads * E : 0);
            long long tp = (HW + cap - 1) / cap;
            long long TL = (HW + tp - 1) / tp;
            TL = (TL + gran - 1) / gran * gran;
            tp = (HW + TL - 1) / TL;
            if (big && (long long)N * tp > kFusedMaxRowsBig) continue;
            if ((long long)N * tp > kFusedMaxRows) return;
            f->big = big;
            f->tp = (int)tp;
            f->TL = (int)TL;
            f->U = (int)(N * tp);
            f->rows = f->U;
            f->rps = (int)(ips * tp);
            // a plane of at most half the slots: the same channel's planes of two consecutive images per unit
            const long long unit_slots = R + (LB == 16 ? lw / W : 0);
            const long long plane_slots = (HW * eb + (long long)kThreads * LB - 1) / ((long long)kThreads * LB);
            if (LB == 16 && tp == 1 && N >= 2 && 2 * plane_slots <= unit_slots && (long long)C * HW * eb <= 0xffffffffLL) {
                f->LPPC = -2;
                f->U = (N + 1) / 2;
                f->rows = N;
                f->rps = ips;
            }
            break;
        }
    }
    // Three or four whole planes per workgroup in workgroup-wide slots, where the layout chosen above is one of the
    // large-plane ones (a tile or two planes per workgroup) and leaves the unit markedly emptier (measured, 64 x 256
    // planes of 100 x 100 floats forward 298 -> 284 us; 128 x 512 planes of 100 x 100 bf16 backward 904 -> 846 us)
    if (f->LPPC <= 0 && LB == 16 && T.big_lds && K <= kFusedMaxShardsBig && N <= kFusedMaxRowsBig && N >= 2 && (long long)C * HW * eb <= 0xffffffffLL) {
        const long long slot_bytes = (long long)kThreads * LB;
        const long long unit_slots = R + lds_words_big / W;                      // of the variant with more unit data in LDS
        const long long plane_bytes = HW * eb, plane_slots = (plane_bytes + slot_bytes - 1) / slot_bytes;
        int best = 0;
        auto consider = [&](int n) { if (unit_slots / n >= plane_slots && n <= N && n > best) best = n; };
#define CGBN_CONSIDER(LB_, LPPC_) consider(-(LPPC_));
        if (forward) { CGBN_FUSED_WGP_FORWARD(CGBN_CONSIDER) } else { CGBN_FUSED_WGP_BACKWARD(CGBN_CONSIDER) }
#undef CGBN_CONSIDER
        // planes a unit holds now
        const double now = f->LPPC == -2 ? 2.0 : 1.0 / (double)(f->tp > 0 ? f->tp : 1);
        if (best > 0 && (double)best >= 1.25 * now && (double)best * (double)plane_bytes >= 0.6 * (double)(unit_slots * slot_bytes)) {
            f->LPPC = -best;
            f->big = 1;
            f->tp = 1;
            f->U = (N + best - 1) / best;
            f->IPU = best;
            f->rows = N;
            f->rps = ips;
        }
    }
    if (f->rows > kFusedMaxRows) return;
    f->total_units = (long long)C * f->U;
    if (f->total_units > 0x7fffffffLL) return;
    int G = 1;
    while (G < kWave && G < f->rps) G <<= 1;
    f->G = G;
    f->ok = 1;
}


// compute units of the current device (256 if there is none to ask)
int compute_units()
{
    static std::mutex lock;
    static std::map<int, int> cache;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 256;
    std::lock_guard<std::mutex> hold(lock);
    auto it = cache.find(dev);
    if (it != cache.end()) return it->second;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) cus = 256;
    cache[dev] = cus;
    return cus;
}

// Pixels per workgroup of the channels-last reduction sweeps.  Measured: these sweeps run
// fastest when the shards are cut into equal pieces and the grid is a whole multiple of the
// compute-unit count (one or two workgroups per unit: 5.7 TB/s against 4.0 with ragged,
// unbalanced pieces), and every further row of partials costs time in the combine step.
// So: the fewest pieces per shard, between 128 KiB and 4 MiB each, that fill the last
// round of workgroups best.
long long reduce_pieces(long long spix, int K, int ctiles, int rpp, long long tile_row_bytes)
{
    const long long quantum = 4LL * rpp;                 // four pixels per thread and pass
    const int cus = compute_units();
    const long long max_pixels = (4LL << 20) / tile_row_bytes > quantum ? (4LL << 20) / tile_row_bytes : quantum;
    const long long first = (spix + max_pixels - 1) / max_pixels;      // fewest pieces of at most 4 MiB
    long long best_pps = first;
    double best = -1.0;
    for (long long pps = first; pps <= first + 2LL * cus; ++pps) {
        long long PL = (spix + pps - 1) / pps;
        PL = (PL + quantum - 1) / quantum * quantum;
        if (PL * tile_row_bytes < (128LL << 10) && pps > first) break;   // too short from here on
        const long long grid = (spix + PL - 1) / PL * K * ctiles;
        const long long rounds = (grid + cus - 1) / cus;
        const double fill = (double)grid / (double)(rounds * cus);
        if (fill > best + 0.02) { best = fill; best_pps = pps; }         // ties go to fewer pieces
        if (fill > 0.98) break;
    }
    long long PL = (spix + best_pps - 1) / best_pps;
    return (PL + quantum - 1) / quantum * quantum;
}

cgbn_status make_plan(const Tuning& T, int N, int C, int H, int W, int layout, int dtype, int K, Plan* p)
{
    if (N < 1 || C < 1 || H < 1 || W < 1) return CGBN_ERR_SHAPE;
    if (layout != CGBN_NCHW && layout != CGBN_NHWC) return CGBN_ERR_ENUM;
    if (dtype != CGBN_F32 && dtype != CGBN_BF16) return CGBN_ERR_ENUM;
    if (K < 1 || K > N || N % K != 0) return CGBN_ERR_SHARD;
    long long HW = (long long)H * W;
    if (HW > 0x3fffffffLL) return CGBN_ERR_SHAPE;
    long long planes = (long long)N * C;
    if (planes > 0x3fffffffLL) return CGBN_ERR_SHAPE;
    long long S = planes * HW;
    if (S > (1LL << 40)) return CGBN_ERR_SHAPE;
    std::memset(p, 0, sizeof(*p));
    p->t = T;
    p->N = N; p->C = C; p->H = H; p->W = W; p->K = K; p->layout = layout; p->dtype = dtype;
    p->eb = dtype == CGBN_F32 ? 4 : 2;
    p->HW = (int)HW;
    p->ips = N / K;
    p->S = S;
    p->M = (double)N * (double)HW;
    const int full_vec = 16 / p->eb;
    if (layout == CGBN_NCHW) {
        p->vec = full_vec;
        if (T.tiny_planes && HW * p->eb <= kTinyPlaneBytes && C % 8 == 0) {
            // several planes of consecutive channels per workgroup: the most that fit the LDS stage, as a power of two
            int tg = 256;
            while (tg > 8 && (long long)tg * HW * p->eb > kTinyStageBytes) tg >>= 1;
            p->tiny = 1;
            p->tg = tg;
            p->L = (int)HW;
            p->sp = 1;
            p->grid = (long long)N * ((C + tg - 1) / tg);
        } else if (HW * p->eb <= T.wave_plane_bytes) {
            p->wave_mode = 1;
            p->L = (int)HW;
            p->sp = 1;
            p->grid = (planes + 3) / 4;
        } else {
            long long L = T.chunk_bytes / p->eb;
            L -= L % (kThreads * full_vec);                    // whole vectors for every thread
            if (L < kThreads * full_vec) L = kThreads * full_vec;
            if (L > HW) L = HW;
            p->L = (int)L;
            p->sp = (int)((HW + L - 1) / L);
            p->grid = planes * p->sp;
        }
        p->rows = N * p->sp;
        p->rps = p->ips * p->sp;
    } else {
        p->vec = (C % full_vec == 0) ? full_vec : 1;
        p->cv = C / p->vec;
        p->TW = p->cv < kThreads ? p->cv : kThreads;
        p->ctiles = (p->cv + p->TW - 1) / p->TW;
        p->rpp = kThreads / p->TW;
        p->spix = (long long)p->ips * HW;
        long long PL;
        if (T.piece_bytes > 0) {
            PL = T.piece_bytes / ((long long)C * p->eb);
            PL -= PL % (4 * p->rpp);                           // four pixels per thread and pass
            if (PL < 4 * p->rpp) PL = 4 * p->rpp;
        } else {
            PL = reduce_pieces(p->spix, K, p->ctiles, p->rpp, (long long)p->TW * p->vec * p->eb);
        }
        if (PL > p->spix) PL = p->spix;
        p->PL = (int)PL;
        long long pps = (p->spix + PL - 1) / PL;
        if (pps * K > 0x3fffffffLL) return CGBN_ERR_SHAPE;
        p->pps = (int)pps;
        p->rows = (int)(pps * K);
        p->rps = (int)pps;
        p->grid = (long long)p->rows * p->ctiles;
        // Pixel runs of the elementwise sweeps.  Measured (fwd normalise / bwd dx, us): bf16 64x50x84x512 64 KiB 186 / 288,
        // 128 KiB 168 / 285, 256 KiB 173 / 296; fp32 16x50x84x1024 32 KiB 175 / 260, 64 KiB 157 / 270, 128 KiB 159 / 274
        // (the same order on 64, 256 and 2048 channels): bf16 128 KiB; fp32 64 KiB with one input tensor, 32 KiB with more.
        for (int two = 0; two < 2; ++two) {
            const long long bytes = T.map_piece_bytes > 0 ? T.map_piece_bytes : p->eb == 2 ? 131072 : two ? 32768 : 65536;
            long long PLm = bytes / ((long long)C * p->eb);
            PLm -= PLm % (4 * p->rpp);
            if (PLm < 4 * p->rpp) PLm = 4 * p->rpp;
            if (PLm > p->spix) PLm = p->spix;
            long long ppsm = (p->spix + PLm - 1) / PLm;
            if (ppsm * K > 0x3fffffffLL) return CGBN_ERR_SHAPE;
            const long long gridm = ppsm * K * p->ctiles;
            if (gridm > 0x7fffffffLL) return CGBN_ERR_SHAPE;
            if (two) { p->PLm2 = (int)PLm; p->ppsm2 = (int)ppsm; p->gridm2 = gridm; }
            else { p->PLm = (int)PLm; p->ppsm = (int)ppsm; p->gridm = gridm; }
        }
    }
    if (p->grid > 0x7fffffffLL || (long long)p->rows * C > (1LL << 33)) return CGBN_ERR_SHAPE;
    int G = 1;
    while (G < kWave && G < p->rps) G <<= 1;
    p->G = G;
    make_fused_plan(T, N, C, HW, K, layout, p->eb, kFusedWords, kFusedLdsWords, kFusedLdsWordsBig, kFusedLdsWordsBigSmall, true, &p->ff);
    make_fused_plan(T, N, C, HW, K, layout, p->eb, kFusedWords / 2, kFusedLdsWords / 2, kFusedLdsWordsBig / 2, kFusedLdsWordsBigSmall / 2, false, &p->fb);
    // Tiny planes that would fill less than half of the register slots a single-launch variant reserves for a plane
    // run faster through the multi-sweep kernels for tiny planes (measured, 256 images, fwd / bwd us: fp32 7x7 x 1024
    // channels 46 / 58 against 132 / 105; bf16 14x14 x 1024 channels, forward, 85 against 126.  Half full, fp32
    // 14x14: level at 256 channels, the single launch ahead at 1024, 131 / 195 against 153 / 222)
    if (p->tiny) {
        for (FusedPlan* f : {&p->ff, &p->fb})
            if (f->ok && f->LPPC > 0 && 2 * f->LPP < f->LPPC) f->ok = 0;
    }
    int max_rows = p->rows;
    if (p->ff.ok && p->ff.rows > max_rows) max_rows = p->ff.rows;
    if (p->fb.ok && p->fb.rows > max_rows) max_rows = p->fb.rows;
    // the sync area comes first, so that the error word has the same offset in every workspace
    size_t sync = align256(((size_t)kSyncHeader + 4 * (size_t)C) * sizeof(unsigned));
    size_t part = align256((size_t)C * max_rows * sizeof(float));
    size_t sh = align256((size_t)K * C * sizeof(double));
    p->off_sync = 0;
    p->off_part0 = sync;
    p->off_part1 = sync + part;
    p->off_sh0 = sync + 2 * part;
    p->off_sh1 = sync + 2 * part + sh;
    p->off_mlo = sync + 2 * part + 2 * sh;
    p->bytes = p->off_mlo + align256((size_t)C * sizeof(float));
    return CGBN_OK;
}

bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

cgbn_status check_ws(const Plan& p, const void* ws, size_t bytes)
{
    if (!ws || ((uintptr_t)ws & 255u) != 0 || bytes < p.bytes) return CGBN_ERR_WORKSPACE;
    return CGBN_OK;
}

cgbn_status launched()
{
    return hipGetLastError() == hipSuccess ? CGBN_OK : CGBN_ERR_HIP;
}

SweepArgs sweep_args(const Plan& p)
{
    SweepArgs A;
    std::memset(&A, 0, sizeof(A));
    A.S = p.S; A.N = p.N; A.C = p.C; A.HW = p.HW; A.rows = p.rows;
    A.L = p.L; A.sp = p.sp;
    A.cv = p.cv; A.TW = p.TW; A.ctiles = p.ctiles; A.rpp = p.rpp; A.PL = p.PL; A.pps = p.pps;
    A.spix = p.spix;
    A.tg = p.tg;
    A.pivot_stride = p.layout == CGBN_NCHW ? p.HW : 1;
    A.inv_M = (float)(1.0 / p.M);
    A.nt = (int)p.t.nt_store;
    return A;
}

template <typename T, int OP> void launch_reduce_t(const Plan& p, const SweepArgs& A, hipStream_t st)
{
    dim3 grid((unsigned)p.grid), block(kThreads);
    if (p.layout == CGBN_NCHW) {
        if (p.tiny) hipLaunchKernelGGL((nchw_reduce_tiny<T, OP>), grid, block, 0, st, A);
        else if (p.wave_mode) hipLaunchKernelGGL((nchw_reduce_wave<T, OP>), grid, block, 0, st, A);
        else hipLaunchKernelGGL((nchw_reduce_block<T, OP>), grid, block, 0, st, A);
    } else {
        if (p.vec == 1) hipLaunchKernelGGL((nhwc_reduce<T, 1, OP>), grid, block, 0, st, A);
        else hipLaunchKernelGGL((nhwc_reduce<T, Elem<T>::VEC, OP>), grid, block, 0, st, A);
    }
}

template <typename T, int EL> void launch_map_t(const Plan& p, const SweepArgs& A, hipStream_t st)
{
    dim3 block(kThreads);
    if (p.layout == CGBN_NCHW) {
        dim3 grid((unsigned)p.grid);
        if (p.tiny) hipLaunchKernelGGL((nchw_map_tiny<T, EL>), grid, block, 0, st, A);
        else if (p.wave_mode) hipLaunchKernelGGL((nchw_map_wave<T, EL>), grid, block, 0, st, A);
        else hipLaunchKernelGGL((nchw_map_block<T, EL>), grid, block, 0, st, A);
    } else {
        constexpr bool more_inputs = el_has_2(EL) || el_has_3(EL);
        dim3 grid((unsigned)(more_inputs ? p.gridm2 : p.gridm));
        SweepArgs B = A;              // the elementwise sweeps cut the pixel runs their own way
        B.PL = more_inputs ? p.PLm2 : p.PLm;
        B.pps = more_inputs ? p.ppsm2 : p.ppsm;
        if (p.vec == 1) hipLaunchKernelGGL((nhwc_map<T, 1, EL>), grid, block, 0, st, B);
        else hipLaunchKernelGGL((nhwc_map<T, Elem<T>::VEC, EL>), grid, block, 0, st, B);
    }
}

cgbn_status launch_reduce(int op, const Plan& p, const SweepArgs& A, hipStream_t st)
{
    const bool f32 = p.dtype == CGBN_F32;
    switch (op) {
    case OP_SUM:   f32 ? launch_reduce_t<float, OP_SUM>(p, A, st)   : launch_reduce_t<bf16_t, OP_SUM>(p, A, st); break;
    case OP_SQDEV: f32 ? launch_reduce_t<float, OP_SQDEV>(p, A, st) : launch_reduce_t<bf16_t, OP_SQDEV>(p, A, st); break;
    case OP_BWD:   f32 ? launch_reduce_t<float, OP_BWD>(p, A, st)   : launch_reduce_t<bf16_t, OP_BWD>(p, A, st); break;
    case OP_MOMENTS: f32 ? launch_reduce_t<float, OP_MOMENTS>(p, A, st) : launch_reduce_t<bf16_t, OP_MOMENTS>(p, A, st); break;
    default:       f32 ? launch_reduce_t<float, OP_BWD_RELU>(p, A, st) : launch_reduce_t<bf16_t, OP_BWD_RELU>(p, A, st); break;
    }
    return launched();
}

cgbn_status launch_map(int el, const Plan& p, const SweepArgs& A, hipStream_t st)
{
    const bool f32 = p.dtype == CGBN_F32;
    switch (el) {
    case EL_NORM:   f32 ? launch_map_t<float, EL_NORM>(p, A, st)   : launch_map_t<bf16_t, EL_NORM>(p, A, st); break;
    case EL_DX:     f32 ? launch_map_t<float, EL_DX>(p, A, st)     : launch_map_t<bf16_t, EL_DX>(p, A, st); break;
    case EL_FROZEN: f32 ? launch_map_t<float, EL_FROZEN>(p, A, st) : launch_map_t<bf16_t, EL_FROZEN>(p, A, st); break;
    case EL_NORM_RELU: f32 ? launch_map_t<float, EL_NORM_RELU>(p, A, st) : launch_map_t<bf16_t, EL_NORM_RELU>(p, A, st); break;
    case EL_NORM_ADD_RELU: f32 ? launch_map_t<float, EL_NORM_ADD_RELU>(p, A, st) : launch_map_t<bf16_t, EL_NORM_ADD_RELU>(p, A, st); break;
    case EL_DX_RELU: f32 ? launch_map_t<float, EL_DX_RELU>(p, A, st) : launch_map_t<bf16_t, EL_DX_RELU>(p, A, st); break;
    default:        f32 ? launch_map_t<float, EL_SCALE>(p, A, st)  : launch_map_t<bf16_t, EL_SCALE>(p, A, st); break;
    }
    return launched();
}

// `pivot_x`: the activation tensor when the rows hold sums about the channel pivots
// (the plain-sum sweep), else null.
cgbn_status launch_combine(int mode, const Plan& p, char* ws, float* out0, float* out1, float* out2,
                           double* sh0, double* sh1, double eps, const void* pivot_x, hipStream_t st,
                           float* out3 = nullptr)
{
    CombineArgs A;
    std::memset(&A, 0, sizeof(A));
    A.part0 = reinterpret_cast<const float*>(ws + p.off_part0);
    A.part1 = reinterpret_cast<const float*>(ws + p.off_part1);
    A.sh0 = sh0; A.sh1 = sh1;
    A.out0 = out0; A.out1 = out1; A.out2 = out2; A.out3 = out3;
    A.M = p.M; A.eps = eps;
    A.shard_count = p.M / p.K;
    A.x = pivot_x;
    A.pivot_stride = pivot_x ? (p.layout == CGBN_NCHW ? p.HW : 1) : 0;
    A.is_bf16 = p.dtype == CGBN_BF16;
    A.C = p.C; A.rows = p.rows; A.K = p.K; A.rps = p.rps; A.G = p.G;
    if (p.layout == CGBN_NCHW) { A.cs = p.rows; A.rs = 1; } else { A.cs = 1; A.rs = p.C; }
    A.clear_word = reinterpret_cast<unsigned*>(ws + p.off_sync) + 1;
    // values per row partial: a chunk of a plane (the last chunk shorter), a whole plane, or a pixel run of a shard
    if (p.layout == CGBN_NCHW) { A.row_mod = p.sp; A.row_full = (p.wave_mode || p.tiny) ? p.HW : p.L; A.row_total = p.HW; }
    else { A.row_mod = p.pps; A.row_full = p.PL; A.row_total = p.spix; }
    dim3 block(kThreads);
    if (p.layout == CGBN_NHWC) {       // a row's channels side by side: 16 channels per workgroup
        constexpr int RL = kThreads / kCombineChannels;
        int G = 1;                     // row lanes per shard: as many as the shard count and a shard's rows allow
        while (2 * G * p.K <= RL && 2 * G <= p.rps) G <<= 1;
        A.G = G;
        dim3 grid((unsigned)((p.C + kCombineChannels - 1) / kCombineChannels));
        switch (mode) {
        case CM_MEAN:   hipLaunchKernelGGL((combine_rows_cl<CM_MEAN>), grid, block, 0, st, A); break;
        case CM_INVSTD: hipLaunchKernelGGL((combine_rows_cl<CM_INVSTD>), grid, block, 0, st, A); break;
        case CM_BWD:    hipLaunchKernelGGL((combine_rows_cl<CM_BWD>), grid, block, 0, st, A); break;
        case CM_SHARDS2: hipLaunchKernelGGL((combine_rows_cl<CM_SHARDS2>), grid, block, 0, st, A); break;
        case CM_MOMENTS: hipLaunchKernelGGL((combine_rows_cl<CM_MOMENTS>), grid, block, 0, st, A); break;
        default:        hipLaunchKernelGGL((combine_rows_cl<CM_SHARDS1>), grid, block, 0, st, A); break;
        }
        return launched();
    }
    dim3 grid((unsigned)((p.C + 3) / 4));
    switch (mode) {
    case CM_MEAN:   hipLaunchKernelGGL((combine_rows<CM_MEAN>), grid, block, 0, st, A); break;
    case CM_INVSTD: hipLaunchKernelGGL((combine_rows<CM_INVSTD>), grid, block, 0, st, A); break;
    case CM_BWD:    hipLaunchKernelGGL((combine_rows<CM_BWD>), grid, block, 0, st, A); break;
    case CM_SHARDS2: hipLaunchKernelGGL((combine_rows<CM_SHARDS2>), grid, block, 0, st, A); break;
    case CM_MOMENTS: hipLaunchKernelGGL((combine_rows<CM_MOMENTS>), grid, block, 0, st, A); break;
    default:        hipLaunchKernelGGL((combine_rows<CM_SHARDS1>), grid, block, 0, st, A); break;
    }
    return launched();
}

// ---- register-resident path ------------------------------------------------

// workgroups of `kernel` that are resident at once on the current device (cached per kernel and device)
template <typename KernelT> int resident_groups(KernelT kernel)
{
    static std::mutex lock;
    static std::map<std::pair<const void*, int>, int> cache;
    int dev = 0, per_cu = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    const std::pair<const void*, int> key(reinterpret_cast<const void*>(kernel), dev);
    std::lock_guard<std::mutex> hold(lock);
    auto it = cache.find(key);
    if (it != cache.end()) return it->second;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, kThreads, 0) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
    cache[key] = per_cu * cus;
    return per_cu * cus;
}

// Start-up stagger of the persistent grid.  All workgroups starting at once run in lock step: every
// channel in flight loads, hands over and writes out at the same time, so the memory system sees a
// read burst, a pause and a write burst per round, and a channel's units, competing with all the
// others, arrive spread out and wait for their last sibling.  Delaying the channel slots class by
// class interleaves those phases.  Measured over 28 launches of 1.3 to 43 rounds (rounds of 23 to
// 61 us): a spread of about 14 us between the first and the last class is at or near the best for
// every launch of at least 4 rounds (forward 2-6 % faster than starting at once, backward 0-6 %);
// spreads proportional to the round are worse at one end or the other, and launches of fewer rounds
// gain nothing or lose what the delay costs, since it is paid once per launch.
// `moved_bytes`: what the launch reads and writes.
void choose_stagger(const Tuning& T, const FusedPlan& f, long long groups, double moved_bytes, FusedArgs& A)
{
    A.stagger_ticks = 0;
    A.stagger_phases = 1;
    const long long slots = groups / f.U, rounds = f.total_units / groups;
    if (!T.stagger || f.U < 2 || slots < 2) return;
    double spread_us = (double)T.stagger_us;
    if (spread_us <= 0.0) {
        if (rounds < 4) return;
        const double round_us = moved_bytes / (double)f.total_units * (double)groups / 4.5e6;   // at 4.5 TB/s
        spread_us = 0.6 * round_us;                 // (short rounds: tiny units)
        if (spread_us > 14.0) spread_us = 14.0;
    }
    const long long phases = slots < T.stagger_phases ? slots : T.stagger_phases;
    A.stagger_phases = (unsigned)phases;
    A.stagger_ticks = (unsigned)(spread_us * 100.0 / (double)(phases - 1));     // 100 MHz clock
}

template <typename KernelT>
cgbn_status launch_fused_kernel(KernelT kernel, const Tuning& T, const FusedPlan& f, FusedArgs& A, int sync_words,
                                hipStream_t st, bool* taken, double moved_bytes)
{
    long long groups = resident_groups(kernel);
    if (T.fused_groups > 0 && T.fused_groups < groups) groups = T.fused_groups;
    if (groups > f.total_units) groups = f.total_units;
    *taken = false;
    if (groups < 1 || f.U > groups) return CGBN_OK;      // a channel's units must all be resident: other path
    // With few channels in flight, a grid that is not a whole number of channels leaves the
    // units of the straddling channel waiting a full round for their siblings: trim it.
    if (T.fused_groups == 0 && groups / f.U < 8) groups = groups / f.U * f.U;
    *taken = true;
    choose_stagger(T, f, groups, moved_bytes, A);
    if (f.U > 1) {      // a channel's only unit hands nothing over: no rows or counters to prepare
        long long want = (A.row_words + kThreads - 1) / kThreads;
        unsigned init_groups = (unsigned)(want < 1 ? 1 : (want > 2048 ? 2048 : want));
        hipLaunchKernelGGL(fused_init, dim3(init_groups), dim3(kThreads), 0, st, A.sync, sync_words,
                           reinterpret_cast<unsigned*>(A.part0), A.row_words);
    }
    if (f.U > 1 && T.cooperative) {
        // Units wait for sibling units, so the whole grid must be resident at once.  Alone on the device it
        // is (the grid is sized for that); a cooperative launch makes the runtime guarantee it also when
        // another such launch is in flight on a different stream, where two half-resident grids could
        // otherwise starve each other until their bounded waits give up.
        void* args[] = {static_cast<void*>(&A)};
        if (hipLaunchCooperativeKernel(reinterpret_cast<const void*>(kernel), dim3((unsigned)groups), dim3(kThreads),
                                       args, 0, st) != hipSuccess) {
            (void)hipGetLastError();
            return CGBN_ERR_HIP;
        }
        return CGBN_OK;
    }
    hipLaunchKernelGGL(kernel, dim3((unsigned)groups), dim3(kThreads), 0, st, A);
    return launched();
}

// Which (bytes per access, slots per plane) variants exist for an element type, direction and activation: all of
// the list header's, except that the float ReLU backward is not built with 4-byte accesses (one slot count
// excepted; see CGBN_FUSED_RELU_BWD_F32_NARROW).  A shape whose variant is not built takes the multi-sweep kernels.
template <typename T, bool FWD, int ACT> constexpr bool fused_built(int LB, int LPPC)
{
    if (std::is_same<T, float>::value && !FWD && ACT == 1 && LB == 4) {
        bool built = false;
#define CGBN_IS_BUILT(LB_, LPPC_) built = built || (LB == LB_ && LPPC == LPPC_);
        CGBN_FUSED_RELU_BWD_F32_NARROW(CGBN_IS_BUILT)
#undef CGBN_IS_BUILT
        return built;
    }
    return true;
}

// ACT: 0 plain, 1 ReLU, 2 shortcut + ReLU (forward only)
template <typename T, bool FWD, int ACT>
cgbn_status launch_fused_t(const Tuning& knobs, const FusedPlan& f, FusedArgs& A, int sync_words, hipStream_t st, bool* taken,
                           double moved_bytes)
{
    *taken = false;
    if (f.big && f.LB == 16 && f.LPPC == 0) {
        if constexpr (FWD) return launch_fused_kernel(nchw_fused_forward<T, 16, 0, ACT, 1>, knobs, f, A, sync_words, st, taken, moved_bytes);
        else return launch_fused_kernel(nchw_fused_backward<T, 16, 0, ACT, 1>, knobs, f, A, sync_words, st, taken, moved_bytes);
    }
    if (f.big && f.LB == 16 && f.LPPC == -2) {
        if constexpr (FWD) return launch_fused_kernel(nchw_fused_forward<T, 16, -2, ACT, 1>, knobs, f, A, sync_words, st, taken, moved_bytes);
        else return launch_fused_kernel(nchw_fused_backward<T, 16, -2, ACT, 1>, knobs, f, A, sync_words, st, taken, moved_bytes);
    }
#define CGBN_FUSED_CASE1(LB_, LPPC_)                                                                         \
    if (f.big == 1 && f.LB == LB_ && f.LPPC == LPPC_) {                                                      \
        if constexpr (FWD) return launch_fused_kernel(nchw_fused_forward<T, LB_, LPPC_, ACT, 1>, knobs, f, A, sync_words, st, taken, moved_bytes); \
        else return launch_fused_kernel(nchw_fused_backward<T, LB_, LPPC_, ACT, 1>, knobs, f, A, sync_words, st, taken, moved_bytes); \
    }
    if constexpr (FWD) {
        CGBN_FUSED_WGP_FORWARD(CGBN_FUSED_CASE1)
    } else {
        CGBN_FUSED_WGP_BACKWARD(CGBN_FUSED_CASE1)
    }
#undef CGBN_FUSED_CASE1
#define CGBN_FUSED_CASE2(LB_, LPPC_)                                                                         \
    if constexpr (fused_built<T, FWD, ACT>(LB_, LPPC_))                                                      \
    if (f.big == 2 && f.LB == LB_ && f.LPPC == LPPC_) {                                                      \
        if constexpr (FWD) return launch_fused_kernel(nchw_fused_forward<T, LB_, LPPC_, ACT, 2>, knobs, f, A, sync_words, st, taken, moved_bytes); \
        else return launch_fused_kernel(nchw_fused_backward<T, LB_, LPPC_, ACT, 2>, knobs, f, A, sync_words, st, taken, moved_bytes); \
    }
    CGBN_FUSED_BIG_SMALL(CGBN_FUSED_CASE2)
#undef CGBN_FUSED_CASE2
#define CGBN_FUSED_CASE(LB_, LPPC_)                                                                          \
    if constexpr (fused_built<T, FWD, ACT>(LB_, LPPC_))                                                      \
    if (f.LB == LB_ && f.LPPC == LPPC_) {                                                                    \
        if constexpr (FWD) return launch_fused_kernel(nchw_fused_forward<T, LB_, LPPC_, ACT, 0>, knobs, f, A, sync_words, st, taken, moved_bytes); \
        else return launch_fused_kernel(nchw_fused_backward<T, LB_, LPPC_, ACT, 0>, knobs, f, A, sync_words, st, taken, moved_bytes); \
    }
    CGBN_FUSED_COMMON(CGBN_FUSED_CASE)
    if constexpr (FWD) {
        CGBN_FUSED_FORWARD_ONLY(CGBN_FUSED_CASE)
    } else {
        CGBN_FUSED_BACKWARD_ONLY(CGBN_FUSED_CASE)
    }
#undef CGBN_FUSED_CASE
    return CGBN_OK;
}

FusedArgs fused_args(const Plan& p, const FusedPlan& f, char* ws)
{
    FusedArgs A;
    std::memset(&A, 0, sizeof(A));
    A.part0 = reinterpret_cast<float*>(ws + p.off_part0);
    A.part1 = reinterpret_cast<float*>(ws + p.off_part1);
    A.sh0 = reinterpret_cast<double*>(ws + p.off_sh0);
    A.sh1 = reinterpret_cast<double*>(ws + p.off_sh1);
    A.sync = reinterpret_cast<unsigned*>(ws + p.off_sync);
    A.row_words = (long long)((p.off_sh0 - p.off_part0) / sizeof(float));   // part0 and part1 are adjacent
    A.total_units = f.total_units;
    A.M = p.M; A.inv_M_f64 = 1.0 / p.M; A.shard_count = p.M / p.K; A.inv_M = (float)(1.0 / p.M);
    A.N = p.N; A.C = p.C; A.HW = p.HW; A.rows = f.rows; A.K = p.K; A.rps = f.rps; A.G = f.G;
    A.U = f.U; A.tp = f.tp; A.TL = f.TL; A.LPP = f.LPP; A.IPU = f.IPU;
    A.nt = (int)p.t.nt_store;
    A.spin_limit = (unsigned)p.t.spin_limit;
    A.wait_ticks = (unsigned long long)p.t.wait_us * 100ull;          // the wall clock counts at 100 MHz
    A.plane_stride = (unsigned)((long long)p.C * p.HW * p.eb);
#ifdef CGBN_TRACE
    A.trace = g_trace;
#endif
    return A;
}

bool eps_ok(float eps) { return std::isfinite(eps) && eps > 0.f; }

#define CGBN_TRY(expr) do { cgbn_status s_ = (expr); if (s_ != CGBN_OK) return s_; } while (0)

}  // namespace

// ===========================================================================
// C ABI
// ===========================================================================

extern "C" {

size_t cgbn_workspace_bytes(int N, int C, int H, int W, cgbn_layout layout, cgbn_dtype dtype, int K)
{
    Plan p;
    if (make_plan(tuning_now(), N, C, H, W, (int)layout, (int)dtype, K, &p) != CGBN_OK) return 0;
    return p.bytes;
}

size_t cgbn_workspace_error_offset(int N, int C, int H, int W, cgbn_layout layout, cgbn_dtype dtype, int K)
{
    Plan p;
    if (make_plan(tuning_now(), N, C, H, W, (int)layout, (int)dtype, K, &p) != CGBN_OK) return (size_t)-1;
    return kErrorWordOffset;
}

cgbn_status cgbn_shard_sum(const void* x, int N, int C, int H, int W, cgbn_layout layout, int K,
                           cgbn_dtype dtype, double* s, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!x || !s) return CGBN_ERR_NULL;
    Plan p;
    CGBN_TRY(make_plan(tuning_now(), N, C, H, W, (int)layout, (int)dtype, K, &p));
    if (!aligned16(x)) return CGBN_ERR_ALIGN;
    CGBN_TRY(check_ws(p, workspace, workspace_bytes));
    char* ws = static_cast<char*>(workspace);
    hipStream_t st = static_cast<hipStream_t>(stream);
    SweepArgs A = sweep_args(p);
    A.x = x;
    A.part0 = reinterpret_cast<float*>(ws + p.off_part0);
    CGBN_TRY(launch_reduce(OP_SUM, p, A, st));
    return launch_combine(CM_SHARDS1, p, ws, nullptr, nullptr, nullptr, s, nullptr, 0.0, x, st);
}

cgbn_status cgbn_reduce_mean(const double* s, int K, int C, long long M, float* mean, float* mean_lo, void* stream)
{
    if (!s || !mean) return CGBN_ERR_NULL;
    if (C < 1 || M < 1) return CGBN_ERR_SHAPE;
    if (K < 1) return CGBN_ERR_SHARD;
    dim3 grid((unsigned)((C + kThreads - 1) / kThreads)), block(kThreads);
    hipLaunchKernelGGL((combine_shards<CM_MEAN>), grid, block, 0, static_cast<hipStream_t>(stream),
                       s, (const double*)nullptr, K, C, (double)M, 0.0, mean, mean_lo);
    return launched();
}

cgbn_status cgbn_shard_sqdev(const void* x, int N, int C, int H, int W, cgbn_layout layout, int K,
                             cgbn_dtype dtype, const float* mean, const float* mean_lo, double* v,
                             void* workspace, size_t workspace_bytes, void* stream)
{
    if (!x || !mean || !v) return CGBN_ERR_NULL;
    Plan p;
    CGBN_TRY(make_plan(tuning_now(), N, C, H, W, (int)layout, (int)dtype, K, &p));
    if (!aligned16(x)) return CGBN_ERR_ALIGN;
    CGBN_TRY(check_ws(p, workspace, workspace_bytes));
    char* ws = static_cast<char*>(workspace);
    hipStream_t st = static_cast<hipStream_t>(stream);
    SweepArgs A = sweep_args(p);
    A.x = x; A.mean = mean; A.mean_lo = mean_lo;
    A.part0 = reinterpret_cast<float*>(ws + p.off_part0);
    CGBN_TRY(launch_reduce(OP_SQDEV, p, A, st));
    return launch_combine(CM_SHARDS1, p, ws, nullptr, nullptr, nullptr, v, nullptr, 0.0, nullptr, st);
}

cgbn_status cgbn_reduce_invstd(const double* v, int K, int C, long long M, float eps, float* invstd, void* stream)
{
    if (!v || !invstd) return CGBN_ERR_NULL;
    if (C < 1 || M < 1) return CGBN_ERR_SHAPE;
    if (K < 1) return CGBN_ERR_SHARD;
    if (!eps_ok(eps)) return CGBN_ERR_EPS;
    dim3 grid((unsigned)((C + kThreads - 1) / kThreads)), block(kThreads);
    hipLaunchKernelGGL((combine_shards<CM_INVSTD>), grid, block, 0, static_cast<hipStream_t>(stream),
                       v, (const double*)nullptr, K, C, (double)M, (double)eps, invstd, (float*)nullptr);
    return launched();
}

cgbn_status cgbn_normalize(const void* x, int N, int C, int H, int W, cgbn_layout layout, cgbn_dtype dtype,
                           const float* mean, const float* mean_lo, const float* invstd,
                           const float* gamma, const float* beta, void* y, void* stream)
{
    if (!x || !mean || !invstd || !gamma || !beta || !y) return CGBN_ERR_NULL;
    Plan p;
    CGBN_TRY(make_plan(tuning_now(), N, C, H, W, (int)layout, (int)dtype, 1, &p));
    if (!aligned16(x) || !aligned16(y)) return CGBN_ERR_ALIGN;
    SweepArgs A = sweep_args(p);
    A.x = x; A.out = y; A.mean = mean; A.mean_lo = mean_lo; A.invstd = invstd; A.gamma = gamma; A.beta = beta;
    return launch_map(EL_NORM, p, A, static_cast<hipStream_t>(stream));
}

cgbn_status cgbn_backward_shard_sums(const void* dy, const void* x, int N, int C, int H, int W,
                                     cgbn_layout layout, int K, cgbn_dtype dtype,
                                     const float* mean, const float* mean_lo, const float* invstd,
                                     double* a, double* b, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!dy || !x || !mean || !invstd || !a || !b) return CGBN_ERR_NULL;
    Plan p;
    CGBN_TRY(make_plan(tuning_now(), N, C, H, W, (int)layout, (int)dtype, K, &p));
    if (!aligned16(x) || !aligned16(dy)) return CGBN_ERR_ALIGN;
    CGBN_TRY(check_ws(p, workspace, workspace_bytes));
    char* ws = static_cast<char*>(workspace);
    hipStream_t st = static_cast<hipStream_t>(stream);
    SweepArgs A = sweep_args(p);
    A.x = x; A.dy = dy; A.mean = mean; A.mean_lo = mean_lo; A.invstd = invstd;
    A.part0 = reinterpret_cast<float*>(ws + p.off_part0);
    A.part1 = reinterpret_cast<float*>(ws + p.off_part1);
    CGBN_TRY(launch_reduce(OP_BWD, p, A, st));
    return launch_combine(CM_SHARDS2, p, ws, nullptr, nullptr, nullptr, a, b, 0.0, nullptr, st);
}

cgbn_status cgbn_backward_reduce(const double* a, const double* b, int K, int C,
                                 float* dbeta, float* dgamma, void* stream)
{
    if (!a || !b || !dbeta || !dgamma) return CGBN_ERR_NULL;
    if (C < 1) return CGBN_ERR_SHAPE;
    if (K < 1) return CGBN_ERR_SHARD;
    dim3 grid((unsigned)((C + kThreads - 1) / kThreads)), block(kThreads);
    hipLaunchKernelGGL((combine_shards<CM_BWD>), grid, block, 0, static_cast<hipStream_t>(stream),
                       a, b, K, C, 1.0, 0.0, dbeta, dgamma);
    return launched();
}

cgbn_status cgbn_backward_dx(const void* dy, const void* x, int N, int C, int H, int W,
                             cgbn_layout layout, cgbn_dtype dtype,
                             const float* mean, const float* mean_lo, const float* invstd,
                             const float* gamma, const float* dgamma, const float* dbeta,
                             void* dx, void* stream)
{
    if (!dy || !x || !mean || !invstd || !gamma || !dgamma || !dbeta || !dx) return CGBN_ERR_NULL;
    Plan p;
    CGBN_TRY(make_plan(tuning_now(), N, C, H, W, (int)layout, (int)dtype, 1, &p));
    if (!aligned16(x) || !aligned16(dy) || !aligned16(dx)) return CGBN_ERR_ALIGN;
    SweepArgs A = sweep_args(p);
    A.x = x; A.dy = dy; A.out = dx; A.mean = mean; A.mean_lo = mean_lo; A.invstd = invstd;
    A.gamma = gamma; A.dgamma = dgamma; A.dbeta = dbeta;
    return launch_map(EL_DX, p, A, static_cast<hipStream_t>(stream));
}

cgbn_status cgbn_frozen_forward(const void* x, int N, int C, int H, int W, cgbn_layout layout, cgbn_dtype dtype,
                                const float* fixed_mean, const float* fixed_var,
                                const float* gamma, const float* beta, float eps, void* y, void* stream)
{
    if (!x || !fixed_mean || !fixed_var || !gamma || !beta || !y) return CGBN_ERR_NULL;
    Plan p;
    CGBN_TRY(make_plan(tuning_now(), N, C, H, W, (int)layout, (int)dtype, 1, &p));
    if (!eps_ok(eps)) return CGBN_ERR_EPS;
    if (!aligned16(x) || !aligned16(y)) return CGBN_ERR_ALIGN;
    SweepArgs A = sweep_args(p);
    A.x = x; A.out = y; A.mean = fixed_mean; A.invstd = fixed_var; A.gamma = gamma; A.beta = beta; A.eps = eps;
    return launch_map(EL_FROZEN, p, A, static_cast<hipStream_t>(stream));
}

cgbn_status cgbn_frozen_backward(const void* dy, int N, int C, int H, int W, cgbn_layout layout, cgbn_dtype dtype,
                                 const float* fixed_var, const float* gamma, float eps, void* dx, void* stream)
{
    if (!dy || !fixed_var || !gamma || !dx) return CGBN_ERR_NULL;
    Plan p;
    CGBN_TRY(make_plan(tuning_now(), N, C, H, W, (int)layout, (int)dtype, 1, &p));
    if (!eps_ok(eps)) return CGBN_ERR_EPS;
    if (!aligned16(dy) || !aligned16(dx)) return CGBN_ERR_ALIGN;
    SweepArgs A = sweep_args(p);
    A.x = dy; A.out = dx; A.invstd = fixed_var; A.gamma = gamma; A.eps = eps;
    return launch_map(EL_SCALE, p, A, static_cast<hipStream_t>(stream));
}

cgbn_status cgbn_update_running_stats(const float* mean, const float* mean_lo, const float* invstd, float eps,
                                      long long M, int C, float momentum, int unbiased,
                                      float* running_mean, float* running_var, void* stream)
{
    if (!mean || !invstd || !running_mean || !running_var) return CGBN_ERR_NULL;
    if (C < 1 || M < 1 || (unbiased && M < 2)) return CGBN_ERR_SHAPE;
    if (!eps_ok(eps)) return CGBN_ERR_EPS;
    if (!(momentum >= 0.f && momentum <= 1.f)) return CGBN_ERR_MOMENTUM;
    const double unbias = unbiased ? (double)M / (double)(M - 1) : 1.0;
    dim3 grid((unsigned)((C + kThreads - 1) / kThreads)), block(kThreads);
    hipLaunchKernelGGL(running_update, grid, block, 0, static_cast<hipStream_t>(stream),
                       mean, mean_lo, invstd, (double)eps, unbias, (double)momentum, running_mean, running_var, C);
    return launched();
}

}  // extern "C"

namespace {

// Algorithm 1, optionally followed by "+ shortcut" and a ReLU (relu == true)
cgbn_status forward_impl(const Tuning& T, const void* x, const void* shortcut, bool relu, int N, int C, int H, int W,
                         cgbn_layout layout, int K, const float* gamma, const float* beta, float eps,
                         void* y, float* mean, float* invstd, cgbn_dtype dtype, float* mean_lo,
                         void* workspace, size_t workspace_bytes, void* stream)
{
    if (!x || !gamma || !beta || !y || !mean || !invstd) return CGBN_ERR_NULL;
    Plan p;
    CGBN_TRY(make_plan(T, N, C, H, W, (int)layout, (int)dtype, K, &p));
    if (!eps_ok(eps)) return CGBN_ERR_EPS;
    if (!aligned16(x) || !aligned16(y) || !aligned16(shortcut)) return CGBN_ERR_ALIGN;
    CGBN_TRY(check_ws(p, workspace, workspace_bytes));
    char* ws = static_cast<char*>(workspace);
    hipStream_t st = static_cast<hipStream_t>(stream);
    float* part0 = reinterpret_cast<float*>(ws + p.off_part0);
    double* sh0 = reinterpret_cast<double*>(ws + p.off_sh0);
    float* mlo = reinterpret_cast<float*>(ws + p.off_mlo);
    const int rev = (int)p.t.reverse;

    if (p.t.fused && p.ff.ok) {
        FusedArgs F = fused_args(p, p.ff, ws);
        F.x = x; F.out = y; F.gamma = gamma; F.beta = beta; F.eps = (double)eps; F.aux = shortcut;
        F.mean = mean; F.mean_lo = mlo; F.mean_lo_user = mean_lo; F.invstd = invstd;
        bool taken = false;
        const int sync_words = kSyncHeader + 4 * p.C;
        const bool f32 = p.dtype == CGBN_F32;
        const double moved = (double)p.S * p.eb * (shortcut ? 3.0 : 2.0);
        cgbn_status st_ = relu && shortcut ? (f32 ? launch_fused_t<float, true, 2>(p.t, p.ff, F, sync_words, st, &taken, moved)
                                                  : launch_fused_t<bf16_t, true, 2>(p.t, p.ff, F, sync_words, st, &taken, moved))
                        : relu ? (f32 ? launch_fused_t<float, true, 1>(p.t, p.ff, F, sync_words, st, &taken, moved)
                                      : launch_fused_t<bf16_t, true, 1>(p.t, p.ff, F, sync_words, st, &taken, moved))
                               : (f32 ? launch_fused_t<float, true, 0>(p.t, p.ff, F, sync_words, st, &taken, moved)
                                      : launch_fused_t<bf16_t, true, 0>(p.t, p.ff, F, sync_words, st, &taken, moved));
        g_last_forward_fused = taken;
        if (taken || st_ != CGBN_OK) return st_;
    }
    g_last_forward_fused = 0;

    SweepArgs A = sweep_args(p);
    A.x = x; A.part0 = part0;
    if (p.t.one_sweep_stats) {
        // Steps 1-10 from ONE sweep over x: every row partial is (sum about the pivot, M2 about the row's own
        // mean); the combine step adds the sums (steps 4-5) and turns the M2s into the squared deviations from
        // the pooled mean by the pairwise update M2 + M2' + (mean' - mean)^2 n n'/(n + n') (steps 6-10: the same
        // number, term for term, as summing (x - mean)^2 directly).  Then step 11: 3 sweeps of the tensor instead of 4.
        A.part1 = reinterpret_cast<float*>(ws + p.off_part1);
        CGBN_TRY(launch_reduce(OP_MOMENTS, p, A, st));
        CGBN_TRY(launch_combine(CM_MOMENTS, p, ws, mean, mlo, mean_lo, nullptr, nullptr, (double)eps, x, st, invstd));
        A.mean = mean; A.mean_lo = mlo; A.invstd = invstd; A.gamma = gamma; A.beta = beta; A.out = y;
        A.reverse = rev; A.dy = shortcut;
        return launch_map(!relu ? EL_NORM : shortcut ? EL_NORM_ADD_RELU : EL_NORM_RELU, p, A, st);
    }
    // steps 1-3 then 4-5
    CGBN_TRY(launch_reduce(OP_SUM, p, A, st));
    CGBN_TRY(launch_combine(CM_MEAN, p, ws, mean, mlo, mean_lo, sh0, nullptr, 0.0, x, st));
    // steps 6-8 then 9-10
    A.mean = mean; A.mean_lo = mlo; A.reverse = rev;
    CGBN_TRY(launch_reduce(OP_SQDEV, p, A, st));
    CGBN_TRY(launch_combine(CM_INVSTD, p, ws, invstd, nullptr, nullptr, sh0, nullptr, (double)eps, nullptr, st));
    // step 11
    A.invstd = invstd; A.gamma = gamma; A.beta = beta; A.out = y; A.reverse = 0;
    A.dy = shortcut;
    return launch_map(!relu ? EL_NORM : shortcut ? EL_NORM_ADD_RELU : EL_NORM_RELU, p, A, st);
}

// The backward; with `y` (the stored output of the ReLU variant) dy is first masked by y > 0
// and `dshortcut`, if not null, receives the masked dy.
cgbn_status backward_impl(const Tuning& T, const void* dy, const void* y, const void* x, const float* mean, const float* invstd,
                          const float* gamma, void* dx, void* dshortcut, float* dgamma, float* dbeta,
                          int N, int C, int H, int W, cgbn_layout layout, int K,
                          cgbn_dtype dtype, const float* mean_lo,
                          void* workspace, size_t workspace_bytes, void* stream)
{
    if (!dy || !x || !mean || !invstd || !gamma || !dx || !dgamma || !dbeta) return CGBN_ERR_NULL;
    const bool relu = y != nullptr;
    Plan p;
    CGBN_TRY(make_plan(T, N, C, H, W, (int)layout, (int)dtype, K, &p));
    if (!aligned16(x) || !aligned16(dy) || !aligned16(dx) || !aligned16(y) || !aligned16(dshortcut)) return CGBN_ERR_ALIGN;
    if (dshortcut && dshortcut == dx) return CGBN_ERR_ALIAS;
    CGBN_TRY(check_ws(p, workspace, workspace_bytes));
    char* ws = static_cast<char*>(workspace);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int rev = (int)p.t.reverse;

    if (p.t.fused && p.fb.ok) {
        FusedArgs F = fused_args(p, p.fb, ws);
        F.x = x; F.dy = dy; F.out = dx; F.gamma = gamma; F.aux = y; F.out2 = dshortcut;
        F.mean = const_cast<float*>(mean); F.mean_lo = const_cast<float*>(mean_lo);
        F.invstd = const_cast<float*>(invstd); F.dgamma = dgamma; F.dbeta = dbeta;
        bool taken = false;
        const int sync_words = kSyncHeader + 4 * p.C;
        const bool f32 = p.dtype == CGBN_F32;
        const double moved = (double)p.S * p.eb * (3.0 + (relu ? 1.0 : 0.0) + (dshortcut ? 1.0 : 0.0));
        cgbn_status st_ = relu ? (f32 ? launch_fused_t<float, false, 1>(p.t, p.fb, F, sync_words, st, &taken, moved)
                                      : launch_fused_t<bf16_t, false, 1>(p.t, p.fb, F, sync_words, st, &taken, moved))
                               : (f32 ? launch_fused_t<float, false, 0>(p.t, p.fb, F, sync_words, st, &taken, moved)
                                      : launch_fused_t<bf16_t, false, 0>(p.t, p.fb, F, sync_words, st, &taken, moved));
        g_last_backward_fused = taken;
        if (taken || st_ != CGBN_OK) return st_;
    }
    g_last_backward_fused = 0;

    SweepArgs A = sweep_args(p);
    A.x = x; A.dy = dy; A.mean = mean; A.mean_lo = mean_lo; A.invstd = invstd;
    A.part0 = reinterpret_cast<float*>(ws + p.off_part0);
    A.part1 = reinterpret_cast<float*>(ws + p.off_part1);
    A.reverse = rev;
    A.aux = y; A.out2 = dshortcut;
    CGBN_TRY(launch_reduce(relu ? OP_BWD_RELU : OP_BWD, p, A, st));
    CGBN_TRY(launch_combine(CM_BWD, p, ws, dbeta, dgamma, nullptr,
                            reinterpret_cast<double*>(ws + p.off_sh0), reinterpret_cast<double*>(ws + p.off_sh1),
                            0.0, nullptr, st));
    A.gamma = gamma; A.dgamma = dgamma; A.dbeta = dbeta; A.out = dx; A.reverse = 0;
    return launch_map(relu ? EL_DX_RELU : EL_DX, p, A, st);
}

}  // namespace

extern "C" {

cgbn_status cgbn_forward(const void* x, int N, int C, int H, int W, cgbn_layout layout, int K,
                         const float* gamma, const float* beta, float eps,
                         void* y, float* mean, float* invstd,
                         cgbn_dtype dtype, float* mean_lo,
                         void* workspace, size_t workspace_bytes, void* stream)
{
    return forward_impl(tuning_now(), x, nullptr, false, N, C, H, W, layout, K, gamma, beta, eps, y, mean, invstd, dtype, mean_lo,
                        workspace, workspace_bytes, stream);
}

cgbn_status cgbn_forward_static(const void* x, int N, int C, int H, int W, cgbn_layout layout, int K,
                                const float* gamma, const float* beta, float eps,
                                void* y, float* mean, float* invstd,
                                cgbn_dtype dtype, float* mean_lo, void* stream)
{
    // every argument error is answered before the device is asked for anything
    if (!x || !gamma || !beta || !y || !mean || !invstd) return CGBN_ERR_NULL;
    const Tuning T = tuning_now();
    Plan p;
    CGBN_TRY(make_plan(T, N, C, H, W, (int)layout, (int)dtype, K, &p));
    if (!eps_ok(eps)) return CGBN_ERR_EPS;
    if (!aligned16(x) || !aligned16(y)) return CGBN_ERR_ALIGN;
    if (p.bytes > (size_t)CGBN_STATIC_SCRATCH_BYTES) return CGBN_ERR_SCRATCH;
    void* ws = nullptr;
    CGBN_TRY(scratch_of_current_device(&ws));
    return forward_impl(T, x, nullptr, false, N, C, H, W, layout, K, gamma, beta, eps, y, mean, invstd, dtype, mean_lo,
                        ws, (size_t)CGBN_STATIC_SCRATCH_BYTES, stream);
}

cgbn_status cgbn_backward(const void* dy, const void* x, const float* mean, const float* invstd,
                          const float* gamma, void* dx, float* dgamma, float* dbeta,
                          int N, int C, int H, int W, cgbn_layout layout, int K,
                          cgbn_dtype dtype, const float* mean_lo,
                          void* workspace, size_t workspace_bytes, void* stream)
{
    return backward_impl(tuning_now(), dy, nullptr, x, mean, invstd, gamma, dx, nullptr, dgamma, dbeta, N, C, H, W, layout, K,
                         dtype, mean_lo, workspace, workspace_bytes, stream);
}

cgbn_status cgbn_forward_relu(const void* x, const void* shortcut, int N, int C, int H, int W,
                              cgbn_layout layout, int K, const float* gamma, const float* beta, float eps,
                              void* y, float* mean, float* invstd, cgbn_dtype dtype, float* mean_lo,
                              void* workspace, size_t workspace_bytes, void* stream)
{
    return forward_impl(tuning_now(), x, shortcut, true, N, C, H, W, layout, K, gamma, beta, eps, y, mean, invstd, dtype, mean_lo,
                        workspace, workspace_bytes, stream);
}

cgbn_status cgbn_backward_relu(const void* dy, const void* y, const void* x, const float* mean, const float* invstd,
                               const float* gamma, void* dx, void* dshortcut, float* dgamma, float* dbeta,
                               int N, int C, int H, int W, cgbn_layout layout, int K,
                               cgbn_dtype dtype, const float* mean_lo,
                               void* workspace, size_t workspace_bytes, void* stream)
{
    if (!y) return CGBN_ERR_NULL;
    return backward_impl(tuning_now(), dy, y, x, mean, invstd, gamma, dx, dshortcut, dgamma, dbeta, N, C, H, W, layout, K,
                         dtype, mean_lo, workspace, workspace_bytes, stream);
}

cgbn_status cgbn_workspace_status(const void* workspace, int* gave_up, void* stream)
{
    if (!workspace || !gave_up) return CGBN_ERR_NULL;
    if (((uintptr_t)workspace & 255u) != 0) return CGBN_ERR_WORKSPACE;
    hipLaunchKernelGGL(error_word_to_flag, dim3(1), dim3(kWave), 0, static_cast<hipStream_t>(stream),
                       static_cast<const unsigned*>(workspace), gave_up);
    return launched();
}

const char* cgbn_status_string(cgbn_status status)
{
    switch (status) {
    case CGBN_OK: return "ok";
    case CGBN_ERR_NULL: return "a required pointer is NULL";
    case CGBN_ERR_SHAPE: return "a dimension is < 1 or the tensor is too large";
    case CGBN_ERR_SHARD: return "need 1 <= K <= N and N % K == 0";
    case CGBN_ERR_ENUM: return "layout or dtype out of range";
    case CGBN_ERR_EPS: return "eps must be finite and > 0";
    case CGBN_ERR_WORKSPACE: return "workspace is NULL, not 256-byte aligned or too small";
    case CGBN_ERR_ALIGN: return "activation tensors must be 16-byte aligned";
    case CGBN_ERR_HIP: return "the HIP runtime refused a launch";
    case CGBN_ERR_TUNING: return "unknown tuning key or value out of range";
    case CGBN_ERR_MOMENTUM: return "momentum outside [0, 1]";
    case CGBN_ERR_ALIAS: return "two outputs that must differ are the same buffer";
    case CGBN_ERR_SCRATCH: return "the problem needs more scratch than the library's static array holds";
    }
    return "unknown status";
}

static long long* tuning_slot(const char* key)
{
    if (!key) return nullptr;
    if (!std::strcmp(key, "chunk_bytes")) return &g_tune.chunk_bytes;
    if (!std::strcmp(key, "wave_plane_bytes")) return &g_tune.wave_plane_bytes;
    if (!std::strcmp(key, "tiny_planes")) return &g_tune.tiny_planes;
    if (!std::strcmp(key, "piece_bytes")) return &g_tune.piece_bytes;
    if (!std::strcmp(key, "map_piece_bytes")) return &g_tune.map_piece_bytes;
    if (!std::strcmp(key, "reverse")) return &g_tune.reverse;
    if (!std::strcmp(key, "nt_store")) return &g_tune.nt_store;
    if (!std::strcmp(key, "fused")) return &g_tune.fused;
    if (!std::strcmp(key, "spin_limit")) return &g_tune.spin_limit;
    if (!std::strcmp(key, "fused_groups")) return &g_tune.fused_groups;
    if (!std::strcmp(key, "one_sweep_stats")) return &g_tune.one_sweep_stats;
    if (!std::strcmp(key, "cooperative")) return &g_tune.cooperative;
    if (!std::strcmp(key, "big_lds")) return &g_tune.big_lds;
    if (!std::strcmp(key, "stagger")) return &g_tune.stagger;
    if (!std::strcmp(key, "stagger_us")) return &g_tune.stagger_us;
    if (!std::strcmp(key, "stagger_phases")) return &g_tune.stagger_phases;
    if (!std::strcmp(key, "wait_us")) return &g_tune.wait_us;
    return nullptr;
}

cgbn_status cgbn_set_tuning(const char* key, long long value)
{
    long long* slot = tuning_slot(key);
    if (!slot) return CGBN_ERR_TUNING;
    if (slot == &g_tune.reverse || slot == &g_tune.nt_store || slot == &g_tune.fused || slot == &g_tune.one_sweep_stats ||
        slot == &g_tune.cooperative || slot == &g_tune.big_lds || slot == &g_tune.stagger || slot == &g_tune.tiny_planes) {
        if (value != 0 && value != 1) return CGBN_ERR_TUNING;
    } else if (slot == &g_tune.spin_limit) {
        if (value < 0 || value > 0xffffffffLL) return CGBN_ERR_TUNING;
    } else if (slot == &g_tune.stagger_us) {
        if (value < 0 || value > 1000) return CGBN_ERR_TUNING;
    } else if (slot == &g_tune.stagger_phases) {
        if (value < 2 || value > 64) return CGBN_ERR_TUNING;
    } else if (slot == &g_tune.wait_us) {
        if (value < 1 || value > 60000000LL) return CGBN_ERR_TUNING;
    } else if (slot == &g_tune.fused_groups) {
        if (value < 0 || value > (1LL << 20)) return CGBN_ERR_TUNING;
    } else if (slot == &g_tune.wave_plane_bytes) {
        if (value < 0 || value > (1LL << 20)) return CGBN_ERR_TUNING;
    } else if ((slot == &g_tune.piece_bytes || slot == &g_tune.map_piece_bytes) && value == 0) {
        // chosen per shape
    } else if (value < 4096 || value > (1LL << 26)) {
        return CGBN_ERR_TUNING;
    }
    std::lock_guard<std::mutex> hold(g_tune_lock);
    *slot = value;
    return CGBN_OK;
}

#ifdef CGBN_TRACE
// performance-work builds only: device buffer of 8 timestamps per unit
void cgbn_debug_set_trace(void* device_buffer) { g_trace = static_cast<unsigned long long*>(device_buffer); }
#endif

cgbn_status cgbn_calibration_copy(const void* src, void* dst, size_t bytes, void* stream)
{
    if (!src || !dst) return CGBN_ERR_NULL;
    if (bytes == 0 || bytes % 16 != 0 || bytes > ((size_t)1 << 40)) return CGBN_ERR_SHAPE;
    if (!aligned16(src) || !aligned16(dst)) return CGBN_ERR_ALIGN;
    const size_t nvec = bytes / 16, per_group = (size_t)kThreads * 8;
    hipLaunchKernelGGL(calibration_copy, dim3((unsigned)((nvec + per_group - 1) / per_group)), dim3(kThreads), 0,
                       static_cast<hipStream_t>(stream), static_cast<const u32x4*>(src), static_cast<u32x4*>(dst), nvec);
    return launched();
}

long long cgbn_plan_get(int N, int C, int H, int W, cgbn_layout layout, cgbn_dtype dtype, int K, const char* key)
{
    Plan p;
    if (!key || make_plan(tuning_now(), N, C, H, W, (int)layout, (int)dtype, K, &p) != CGBN_OK) return -1;
    const bool bwd = !std::strncmp(key, "bwd_", 4);
    if (bwd || !std::strncmp(key, "fwd_", 4)) {
        const FusedPlan& f = bwd ? p.fb : p.ff;
        const char* k = key + 4;
        if (!std::strcmp(k, "ok")) return f.ok;
        if (!std::strcmp(k, "LB")) return f.LB;
        if (!std::strcmp(k, "LPPC")) return f.LPPC;
        if (!std::strcmp(k, "LPP")) return f.LPP;
        if (!std::strcmp(k, "IPU")) return f.IPU;
        if (!std::strcmp(k, "U")) return f.U;
        if (!std::strcmp(k, "tp")) return f.tp;
        if (!std::strcmp(k, "TL")) return f.TL;
        if (!std::strcmp(k, "rows")) return f.rows;
        if (!std::strcmp(k, "rps")) return f.rps;
        if (!std::strcmp(k, "G")) return f.G;
        if (!std::strcmp(k, "big")) return f.big;
        if (!std::strcmp(k, "total_units")) return f.total_units;
        return -1;
    }
    if (!std::strcmp(key, "wave_mode")) return p.wave_mode;
    if (!std::strcmp(key, "tiny")) return p.tiny;
    if (!std::strcmp(key, "tg")) return p.tg;
    if (!std::strcmp(key, "L")) return p.L;
    if (!std::strcmp(key, "sp")) return p.sp;
    if (!std::strcmp(key, "vec")) return p.vec;
    if (!std::strcmp(key, "cv")) return p.cv;
    if (!std::strcmp(key, "TW")) return p.TW;
    if (!std::strcmp(key, "ctiles")) return p.ctiles;
    if (!std::strcmp(key, "rpp")) return p.rpp;
    if (!std::strcmp(key, "PL")) return p.PL;
    if (!std::strcmp(key, "pps")) return p.pps;
    if (!std::strcmp(key, "PLm")) return p.PLm;
    if (!std::strcmp(key, "ppsm")) return p.ppsm;
    if (!std::strcmp(key, "PLm2")) return p.PLm2;
    if (!std::strcmp(key, "ppsm2")) return p.ppsm2;
    if (!std::strcmp(key, "gridm2")) return p.gridm2;
    if (!std::strcmp(key, "rows")) return p.rows;
    if (!std::strcmp(key, "rps")) return p.rps;
    if (!std::strcmp(key, "G")) return p.G;
    if (!std::strcmp(key, "grid")) return p.grid;
    if (!std::strcmp(key, "gridm")) return p.gridm;
    if (!std::strcmp(key, "part_bytes")) return (long long)(p.off_part1 - p.off_part0);
    if (!std::strcmp(key, "shard_bytes")) return (long long)(p.off_sh1 - p.off_sh0);
    return -1;
}

long long cgbn_get_tuning(const char* key)
{
    if (key && !std::strcmp(key, "last_forward_fused")) return g_last_forward_fused.load();
    if (key && !std::strcmp(key, "last_backward_fused")) return g_last_backward_fused.load();
    long long* slot = tuning_slot(key);
    if (!slot) return -1;
    std::lock_guard<std::mutex> hold(g_tune_lock);
    return *slot;
}

}  // extern "C"
