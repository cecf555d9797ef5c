// AdaScale SGD step for MI355X (gfx950): host side of the C ABI declared in adascale.h, and the
// choice and launch of the kernels (adascale_device.h).
//
// A step never needs the host.  In its general form it is three launches on the caller's stream:
//   reduce  : one streaming pass over the S gradient buffers; writes the mean gradient
//             (Sec. 2, Algorithm 1) and fp64 partial sums of A = sum_i ||g_i||^2 and
//             B = ||gbar||^2 (App. B.3) into slots fixed by the data, not by the scheduling;
//   scalars : one workgroup sums the partials in a fixed order and evaluates the estimates,
//             clamps, moving averages, gain ratio r_t, eta_t and tau (App. B.3, eq. 3, Sec. 3.2);
//   update  : v <- rho v + gbar + lambda w, w <- w - eta_t v with eta_t read from device memory.
// Three implementations exist (adascale_step_path): the fused step, one persistent launch that
// keeps the mean gradient in registers and LDS across a grid barrier (parameter lists up to
// several times the chip's capacity); the three kernels above with a persistent, memory-ordered
// reduce kernel (larger lists); and the three kernels in their general form (any scale).
// The path is bandwidth bound (about half a flop per byte), so there is no matrix-core work:
// the kernels are 8- or 16-byte-per-lane coalesced streams, 64-lane shuffle reductions and fp64
// accumulation of exact squares.

#include "adascale_device.h"

// Defined in fused_level.hip, compiled once per register-slot level and gain variant.
extern "C" {
__attribute__((visibility("hidden"))) const void *adascale_fused_kernel_level0_lag0(int dtype, int S);
__attribute__((visibility("hidden"))) const void *adascale_fused_kernel_level0_lag1(int dtype, int S);
__attribute__((visibility("hidden"))) const void *adascale_fused_kernel_level1_lag0(int dtype, int S);
__attribute__((visibility("hidden"))) const void *adascale_fused_kernel_level1_lag1(int dtype, int S);
__attribute__((visibility("hidden"))) const void *adascale_fused_kernel_level2_lag0(int dtype, int S);
__attribute__((visibility("hidden"))) const void *adascale_fused_kernel_level2_lag1(int dtype, int S);
__attribute__((visibility("hidden"))) const void *adascale_fused_kernel_level3_lag0(int dtype, int S);
__attribute__((visibility("hidden"))) const void *adascale_fused_kernel_level3_lag1(int dtype, int S);
}

namespace {

thread_local char g_init_error[256] = "";

// Last fused launch on each device (see adascale_step).
constexpr int kMaxDevices = 64;
struct FusedChain {
    std::mutex m;
    hipEvent_t ev = nullptr;
    hipStream_t last_stream = nullptr;
    bool used = false;
};
FusedChain g_chain[kMaxDevices];

}  // namespace

// Device memory of adascale_step_flat, the entry point that allocates nothing: one block per GPU,
// held from the moment the library is loaded until the process ends.  In host code this name is
// only a handle for hipGetSymbolAddress (flat_scratch_on); kernels get the address it returns.
static __device__ __align__(256) unsigned char scratch[(sizeof(FlatScratch) + 255) / 256 * 256];

namespace {

std::mutex g_flat_mutex;
FlatScratch *g_flat_scratch[kMaxDevices] = {};  // address of `scratch` on each device, looked up once

}  // namespace

// ---------------------------------------------------------------------------------------------
struct adascale_ctx {
    adascale_config cfg{};
    std::vector<long long> numel;
    std::vector<int> tile_prefix;   // [N+1]
    std::vector<int> span_first;    // [n_spans]
    std::vector<size_t> gbar_off;   // element offset of tensor k in the mean-gradient scratch
    size_t gbar_len = 0;            // its length in elements
    // The full scratch (d elements) is only allocated once a step needs it: the general step and
    // the streaming step without momentum.  Otherwise only the ragged last tiles of the tensors
    // pass through memory, in a scratch of one tile per tensor.
    float *d_cold_gbar = nullptr;
    std::vector<unsigned long long> cold_base;  // per tensor: address that tensor's element 0 would have
    long long d = 0;
    int vec = 4, tile = 1024;
    int n_tiles = 0, span_tiles = 2, n_spans = 0;
    int S_cap = 0;                  // pointer table capacity in replica slots per row
    adascale_tuning tun{};          // knobs of adascale_init_tuned (all zero: the library's choices)
    bool failed = false;            // a fused step's grid barrier gave up (seen by adascale_get_state)
    bool fail_next = false;         // adascale_fail_next_barrier

    int *d_span_first = nullptr, *d_tile_prefix = nullptr;
    long long *d_numel = nullptr;
    // The device keeps the pointer tables of the last kTables distinct pointer sets; table j's
    // pinned host mirror h_tab[j] is also the staging buffer it is uploaded from.
    unsigned long long *d_tab[kTables] = {};
    unsigned long long *h_tab[kTables] = {};
    hipEvent_t tab_ev[kTables] = {};   // upload of table j
    bool tab_uploaded[kTables] = {};   // tab_ev[j] has been recorded
    size_t tab_len[kTables] = {};      // 0: table j holds nothing
    unsigned long long tab_used[kTables] = {};  // step count of the last use (the oldest is replaced)
    unsigned long long steps_issued = 0;
    int tab_last = 0;                  // table of the last step
    bool tab_captured[kTables] = {};   // a captured step refers to table j: it is never replaced
    std::vector<unsigned long long> tab_build;  // the table of the current call
    float *d_gbar = nullptr, *d_lr = nullptr;
    double *d_partials = nullptr;
    // Progress of the context (current state record, barrier generation, fault flag, claim
    // counter): kept on the device and advanced by the kernels, so that the host passes the same
    // arguments at every step and a captured step can be replayed.
    DevBook *d_book = nullptr;

    // fused single-launch path
    std::vector<FTile> ftiles, ctiles;   // full tiles, ragged last tiles
    FTile *d_ftiles = nullptr, *d_ctiles = nullptr;
    int f_grid = 0, f_tpb = 0, f_lds_cap = 0, f_level = 0;
    bool fused_ok = false;

    // streaming reduce (first kernel of the three-kernel step)
    bool tiles_ok = false, stream_ok = false;
    int n_cus = 0, s_grid = 0;
    int s_keep = 0;                      // tiles the streaming sweep keeps in LDS between write bursts
    size_t s_lds = 0;                    // its dynamic LDS
    int wall_khz = 100000;               // rate of the clock the bursts are timed by
    bool stream_momentum = true;         // the sweep writes the new momentum instead of the mean gradient

    DevBook *h_book = nullptr;      // pinned

    std::vector<hipEvent_t> prof_ev;  // 4 per recorded step
    int prof_cap = 0, prof_n = 0;
    bool prof_on = false;

    char err[256] = "";
};

namespace {

int fail(adascale_ctx *c, int code, const char *fmt, ...)
{
    char *dst = c ? c->err : g_init_error;
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(dst, 256, fmt, ap);
    va_end(ap);
    return code;
}

#define HIP_TRY(ctx, call)                                                                         \
    do {                                                                                           \
        hipError_t e_ = (call);                                                                    \
        if (e_ != hipSuccess) return fail(ctx, ADASCALE_EHIP, "%s: %s", #call, hipGetErrorString(e_)); \
    } while (0)

// Makes the context's device current for the duration of a call and puts the caller's back.
struct DeviceGuard {
    int prev = -1;
    bool switched = false;
    hipError_t enter(int device)
    {
        hipError_t e = hipGetDevice(&prev);
        if (e != hipSuccess || prev == device) return e;
        e = hipSetDevice(device);
        switched = e == hipSuccess;
        return e;
    }
    ~DeviceGuard()
    {
        if (switched) (void)hipSetDevice(prev);
    }
};

// Replica slots in a pointer-table row: the 512-lane kernels read whole half-groups, so rows are
// padded to their HG * NH slots (the padding repeats the last replica).
int padded_scale(int dtype, int S);
size_t table_len(const adascale_ctx *c, int S)
{
    return (size_t)c->numel.size() * (size_t)(padded_scale(c->cfg.grad_dtype, S) + kRowG);
}

void forget_tables(adascale_ctx *c)
{
    for (int j = 0; j < kTables; ++j) {
        c->tab_len[j] = 0;
        c->tab_captured[j] = false;  // graphs captured before this point are void (see adascale_step)
    }
}

int alloc_pointer_tables(adascale_ctx *c, int S)
{
    const int slots = padded_scale(c->cfg.grad_dtype, S);
    if (slots <= c->S_cap) return ADASCALE_OK;
    const size_t bytes = std::max<size_t>(table_len(c, S), 1) * sizeof(unsigned long long);
    if (c->d_tab[0]) HIP_TRY(c, hipDeviceSynchronize());  // kernels in flight may still read the old tables
    for (int j = 0; j < kTables; ++j) {
        if (c->d_tab[j]) HIP_TRY(c, hipFree(c->d_tab[j]));
        c->d_tab[j] = nullptr;
        if (c->h_tab[j]) HIP_TRY(c, hipHostFree(c->h_tab[j]));
        c->h_tab[j] = nullptr;
        c->tab_uploaded[j] = false;
    }
    for (int j = 0; j < kTables; ++j) {
        HIP_TRY(c, hipMalloc(&c->d_tab[j], bytes));
        HIP_TRY(c, hipHostMalloc(&c->h_tab[j], bytes, hipHostMallocDefault));
    }
    c->S_cap = slots;
    forget_tables(c);
    return ADASCALE_OK;
}

// Is [p, p + bytes) inside one device allocation on this device?  `lo`/`hi` cache the last range.
bool device_range_ok(const void *p, size_t bytes, int device, uintptr_t &lo, uintptr_t &hi)
{
    const uintptr_t a = (uintptr_t)p;
    if (a >= lo && a + bytes <= hi) return true;
    hipPointerAttribute_t attr;
    if (hipPointerGetAttributes(&attr, p) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    if (attr.type != hipMemoryTypeDevice && attr.type != hipMemoryTypeManaged) return false;
    if (attr.type == hipMemoryTypeDevice && attr.device != device) return false;
    hipDeviceptr_t base = nullptr;
    size_t size = 0;
    if (hipMemGetAddressRange(&base, &size, const_cast<void *>(p)) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    lo = (uintptr_t)base;
    hi = lo + size;
    return a >= lo && a + bytes <= hi;
}

// The fused kernel instance for a gradient type, scale S, register-slot level and gain variant
// (nullptr: none, use the general step), and the number of register slots it keeps.  The
// instances of each level live in a translation unit of their own (fused_level.hip).
const void *fused_kernel_for(int dtype, int S, int level, bool lag, int *regs = nullptr)
{
    int hg = 0, nh = 0;
    if (!fused_shape(dtype, S, &hg, &nh)) return nullptr;
    if (regs) *regs = fused_regs_at(level);
    switch (level) {
    case 0: return lag ? adascale_fused_kernel_level0_lag1(dtype, S) : adascale_fused_kernel_level0_lag0(dtype, S);
    case 1: return lag ? adascale_fused_kernel_level1_lag1(dtype, S) : adascale_fused_kernel_level1_lag0(dtype, S);
    case 2: return lag ? adascale_fused_kernel_level2_lag1(dtype, S) : adascale_fused_kernel_level2_lag0(dtype, S);
    case 3: return lag ? adascale_fused_kernel_level3_lag1(dtype, S) : adascale_fused_kernel_level3_lag0(dtype, S);
    default: return nullptr;
    }
}

// The streaming reduce kernel instance for a gradient type and scale (nullptr: none).
const void *stream_kernel_for(int dtype, int S)
{
#define KS(GT, HG, NH, MASK) reinterpret_cast<const void *>(k_reduce_stream<GT, HG, NH, MASK>)
    int hg = 0, nh = 0;
    if (!fused_shape(dtype, S, &hg, &nh)) return nullptr;
    if (nh != 2 && nh != 4 && nh != 8) return dtype == ADASCALE_F32 ? KS(float, 4, 0, true) : KS(Bf16, 8, 0, true);
    const bool exact = hg * nh == S;
    if (dtype == ADASCALE_F32) {
        switch (hg * 100 + nh) {
        case 102: return exact ? KS(float, 1, 2, false) : KS(float, 1, 2, true);
        case 202: return exact ? KS(float, 2, 2, false) : KS(float, 2, 2, true);
        case 402: return exact ? KS(float, 4, 2, false) : KS(float, 4, 2, true);
        case 404: return exact ? KS(float, 4, 4, false) : KS(float, 4, 4, true);
        case 408: return KS(float, 4, 8, true);
        default: return nullptr;
        }
    }
    switch (hg * 100 + nh) {
    case 102: return KS(Bf16, 1, 2, true);
    case 202: return KS(Bf16, 2, 2, true);
    case 402: return KS(Bf16, 4, 2, true);
    case 802: return KS(Bf16, 8, 2, true);
    case 804: return KS(Bf16, 8, 4, true);
    case 808: return KS(Bf16, 8, 8, true);
    default: return nullptr;
    }
#undef KS
}

// Least dynamic LDS the streaming reduce kernel asks for (its ring of kept tiles may need less):
// more than half a CU's LDS, so that its workgroups (one per CU in number) also land one per CU.
constexpr size_t kStreamLdsPad = 96 * 1024;
constexpr int kFusedMinPct = 8;   // least share of the mean gradient on chip for the fused step

// ---- planning: pure host arithmetic (no HIP calls), shared by the set-up below and adascale_plan ----

// Whole 512-lane tiles (inside one tensor) and ragged last tiles of a parameter list; false if the
// list is outside what the 512-lane kernels index (then the general kernels run).
bool plan_tiles(const long long *numel, int N, long long *full, long long *ragged)
{
    long long nt = 0, nc = 0;
    for (int k = 0; k < N; ++k) {
        if (numel[k] >= (1LL << 40)) return false;
        nt += numel[k] / kFTile;
        if (nt > 0x3fffffffLL) return false;
        if (numel[k] % kFTile) ++nc;
    }
    *full = nt;
    *ragged = nc;
    return true;
}

// Length of the clock windows in which a sweep writes its kept tiles (BurstRing), in ticks of the
// device's wall clock: 0.8 of the time a workgroup takes to fill a ring of `keep` tiles when
// `grid` workgroups sweep at 6.5 TB/s together, so that the ring is rarely full before a window
// opens.  Returned as 2^64 / ticks, the factor the kernel turns a clock reading into a window
// number with; 0 (no bursts) if there is no ring.
unsigned long long burst_window_factor(const adascale_ctx *c, int S, int grid, int keep, double min_grad_bytes)
{
    if (keep <= 0 || c->tun.burst_tiles < 0) return 0;
    const double b = c->cfg.grad_dtype == ADASCALE_F32 ? 4.0 : 2.0;
    // With few gradient bytes per parameter the writes are too large a share of the sweep to be set
    // apart.  Measured at d = 351 M: on the streaming sweep bursts cost 7-12 % at 2-16 gradient
    // bytes per parameter and gain 0.7 % at 32, 4-7 % at 64, 6 % at 128; on the fused step (9 % on
    // chip) they cost 8 % at 8 bytes and gain 1-7 % at 16, 4-11 % at 24, 11-13 % at 32, 16 % at 128.
    // (A knob that asks for bursts gets them at any scale.)
    if (S * b < min_grad_bytes && c->tun.burst_tiles == 0 && c->tun.burst_window_ticks <= 0) return 0;
    double ticks = (double)c->tun.burst_window_ticks;
    if (ticks <= 0) {
        const double tile_bytes = (double)kFTile * (S * b + (c->cfg.weight_decay != 0.0 ? 12.0 : 8.0));
        const double us_per_tile = tile_bytes * std::max(1, grid) / 6.5e6;
        ticks = 0.8 * keep * us_per_tile * c->wall_khz / 1000.0;
    }
    ticks = std::min(std::max(ticks, 64.0), 1e9);
    return (unsigned long long)(18446744073709551616.0 / ticks);
}

// May the streaming reduce kernel run on this device at all (its grid: plan_stream_grid)?
bool plan_stream_ok(const adascale_tuning &tun, size_t lds_per_workgroup)
{
    if (tun.force_path == ADASCALE_FORCE_GENERAL) return false;
    return lds_per_workgroup >= kStreamLdsPad + 1024;
}

int plan_stream_grid(long long nt, long long nc, int cus)
{
    const long long n_pairs = (nt + 1) / 2;
    return (int)std::max<long long>(1, std::min<long long>(std::max<long long>(n_pairs, nc), std::min(cus, kFMaxGrid)));
}

// The fused step's shape for a parameter list on a device with `cus` compute units and
// `lds_per_workgroup` bytes of LDS: grid (one workgroup per CU), tiles per workgroup, the
// register-slot level, the LDS capacity in tiles, the share of the mean gradient kept on chip.
struct FusedPlan {
    bool ok = false;
    int grid = 0, tpb = 0, level = 0, lds_cap = 0, on_chip_pct = 0;
};

FusedPlan plan_fused(const adascale_tuning &tun, long long nt, long long nc, int cus_of_device, size_t lds_per_workgroup,
                     bool stream_ok)
{
    FusedPlan f;
    if (tun.force_path == ADASCALE_FORCE_GENERAL || tun.force_path == ADASCALE_FORCE_STREAMING) return f;
    if (nt + nc == 0) return f;
    const int cus = std::min(std::min(cus_of_device, kFMaxGrid), tun.fused_max_grid > 0 ? tun.fused_max_grid : kFMaxGrid);
    f.grid = (int)std::max<long long>(1, std::min<long long>(std::max(nt, nc), cus));
    f.tpb = (int)((nt + f.grid - 1) / f.grid);
    f.lds_cap = lds_per_workgroup > 6144 ? (int)((lds_per_workgroup - 6144) / (kFThreads * sizeof(f4))) : 0;  // static LDS is 5.3 KB
    // Register-slot level: among those whose slot count every workgroup can fill, the lowest that,
    // with the LDS, still holds every tile of a workgroup (the registers it leaves free take w and
    // v of more tiles ahead of the grid barrier), else the highest.
    for (int l = 0; l < kFRegLevels; ++l) {
        if (fused_regs_at(l) > nt / f.grid) break;
        f.level = l;
        if (fused_regs_at(l) + f.lds_cap >= f.tpb) break;
    }
    // with very little of the mean gradient on chip the three-kernel step with the streaming reduce
    // kernel takes over (measured on lists of 62 M to 1.06 G parameters: the fused step is the
    // faster one by 1-10 % down to 13 % on chip, the two are within 2 % of each other at 9-10 %,
    // within 3 % either way at 3-5 %, gradients of 32 bytes per parameter and more)
    f.on_chip_pct = f.tpb == 0 ? 100 : std::min(100, 100 * (fused_regs_at(f.level) + std::min(f.tpb, f.lds_cap)) / f.tpb);
    const int min_pct = tun.force_path == ADASCALE_FORCE_FUSED ? 0 : tun.fused_min_percent > 0 ? tun.fused_min_percent : kFusedMinPct;
    if (stream_ok && f.on_chip_pct < min_pct) return f;
    f.ok = true;
    return f;
}

// Tile tables of the 512-lane kernels: whole tiles (inside one tensor) and the ragged last tile
// of each tensor; the streaming reduce kernel's grid and counters.
int setup_tiles(adascale_ctx *c)
{
    c->tiles_ok = c->stream_ok = false;
    if (c->d == 0) return ADASCALE_OK;
    hipDeviceProp_t prop;
    HIP_TRY(c, hipGetDeviceProperties(&prop, c->cfg.device));
    c->n_cus = prop.multiProcessorCount;
    {
        int khz = 0;  // the clock the write bursts are timed by
        if (hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, c->cfg.device) != hipSuccess || khz <= 0) {
            (void)hipGetLastError();
            khz = 100000;
        }
        c->wall_khz = khz;
    }
    const int N = (int)c->numel.size();
    long long full = 0, ragged = 0;
    if (!plan_tiles(c->numel.data(), N, &full, &ragged)) return ADASCALE_OK;
    c->ftiles.clear();
    c->ctiles.clear();
    for (int k = 0; k < N; ++k) {
        const long long nf = c->numel[k] / kFTile;
        for (long long j = 0; j < nf; ++j) c->ftiles.push_back(FTile{k, (int)j});
        if (c->numel[k] % kFTile) c->ctiles.push_back(FTile{k, (int)nf});
    }
    const size_t nt = c->ftiles.size(), nc = c->ctiles.size();
    HIP_TRY(c, hipMalloc(&c->d_ftiles, sizeof(FTile) * std::max<size_t>(nt, 1)));
    HIP_TRY(c, hipMalloc(&c->d_ctiles, sizeof(FTile) * std::max<size_t>(nc, 1)));
    if (nt) HIP_TRY(c, hipMemcpy(c->d_ftiles, c->ftiles.data(), sizeof(FTile) * nt, hipMemcpyHostToDevice));
    if (nc) HIP_TRY(c, hipMemcpy(c->d_ctiles, c->ctiles.data(), sizeof(FTile) * nc, hipMemcpyHostToDevice));
    // scratch for the ragged tiles: tensor k's tile sits at slot j, and the address handed to the
    // kernels is the one element 0 of the tensor would have if the whole tensor were there
    HIP_TRY(c, hipMalloc(&c->d_cold_gbar, sizeof(float) * kFTile * std::max<size_t>(nc, 1)));
    c->cold_base.assign(N, (unsigned long long)(uintptr_t)c->d_cold_gbar);
    for (size_t j = 0; j < nc; ++j) {
        const FTile &t = c->ctiles[j];
        c->cold_base[t.k] = (unsigned long long)(uintptr_t)(c->d_cold_gbar + j * kFTile) -
                            (unsigned long long)t.local * kFTile * sizeof(float);
    }
    c->tiles_ok = true;

    if (!plan_stream_ok(c->tun, prop.sharedMemPerBlock)) return ADASCALE_OK;
    c->s_grid = plan_stream_grid((long long)nt, (long long)nc, c->n_cus);
    {
        const int cap = (int)std::min<size_t>(kStreamKeepMax, (prop.sharedMemPerBlock - 2048) / (kFThreads * sizeof(f4)));
        const int want = c->tun.burst_tiles;
        c->s_keep = want < 0 ? 0 : std::min(cap, want > 0 ? want : kStreamKeepMax);
        c->s_lds = std::max(kStreamLdsPad, (size_t)c->s_keep * kFThreads * sizeof(f4));
    }
    const int max_scale = (c->cfg.grad_dtype == ADASCALE_F32 ? kFMaxScaleF32 : kFMaxScaleBf16) + 1;  // + the run-time shape
    for (int S = 1; S <= max_scale; ++S) {
        const void *fn = stream_kernel_for(c->cfg.grad_dtype, S);
        if (fn) HIP_TRY(c, hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)c->s_lds));
    }
    c->stream_momentum = c->tun.stream_via_scratch != 1;
    c->stream_ok = true;
    return ADASCALE_OK;
}

// Decide whether the fused single-launch step applies (plan_fused) and prepare its kernel
// instances.  Which instance runs is looked up per step from the scale of the moment (it may
// change between steps).
int setup_fused(adascale_ctx *c)
{
    c->fused_ok = false;
    if (!c->tiles_ok) return ADASCALE_OK;
    hipDeviceProp_t prop;
    HIP_TRY(c, hipGetDeviceProperties(&prop, c->cfg.device));
    if ((c->cfg.flags & ADASCALE_COOPERATIVE_LAUNCH) && !prop.cooperativeLaunch) return ADASCALE_OK;
    const FusedPlan f = plan_fused(c->tun, (long long)c->ftiles.size(), (long long)c->ctiles.size(),
                                   prop.multiProcessorCount, prop.sharedMemPerBlock, c->stream_ok);
    if (!f.ok) return ADASCALE_OK;
    const size_t lds_bytes = (size_t)f.lds_cap * kFThreads * sizeof(f4);
    const int max_scale = (c->cfg.grad_dtype == ADASCALE_F32 ? kFMaxScaleF32 : kFMaxScaleBf16) + 1;  // + the run-time shape
    for (int S = 1; S <= max_scale; ++S) {
        // with ADASCALE_LAGGED_R either variant may run, depending on the scale of the moment
        for (int lag = 0; lag <= ((c->cfg.flags & ADASCALE_LAGGED_R) ? 1 : 0); ++lag) {
            const void *fn = fused_kernel_for(c->cfg.grad_dtype, S, f.level, lag != 0);
            if (!fn) continue;
            HIP_TRY(c, hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes));
            int per_cu = 0;
            HIP_TRY(c, hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, kFThreads, lds_bytes));
            if (per_cu < 1 || (long long)per_cu * prop.multiProcessorCount < f.grid) return ADASCALE_OK;
        }
    }
    c->f_grid = f.grid;
    c->f_tpb = f.tpb;
    c->f_lds_cap = f.lds_cap;
    c->f_level = f.level;
    c->fused_ok = true;
    return ADASCALE_OK;
}

template <typename GT>
void launch_reduce(const adascale_ctx *c, const unsigned long long *d_ptrs, int grid, hipStream_t s, int S)
{
    const double inv_S = 1.0 / (double)S;
    const int row_len = padded_scale(c->cfg.grad_dtype, S) + kRowG;
#define LAUNCH(HH)                                                                                   \
    hipLaunchKernelGGL((k_reduce<GT, HH>), dim3(grid), dim3(kThreads), 0, s, c->d_span_first,        \
                       c->d_tile_prefix, c->d_numel, d_ptrs, c->d_partials, c->n_tiles,              \
                       c->span_tiles, c->n_spans, S, row_len, inv_S)
    // replicas per half-group (two half-groups in flight)
    if (S >= 16) LAUNCH(8);
    else if (S >= 8) LAUNCH(4);
    else if (S >= 4) LAUNCH(2);
    else LAUNCH(1);
#undef LAUNCH
}

template <typename GT>
void launch_reduce_update(const adascale_ctx *c, const unsigned long long *d_ptrs, int grid, hipStream_t s, int S,
                          const ScalarArgs &sa)
{
    const double inv_S = 1.0 / (double)S;
    const int row_len = padded_scale(c->cfg.grad_dtype, S) + kRowG;
    const float rho = (float)c->cfg.momentum, lambda = (float)c->cfg.weight_decay;
#define LAUNCH(HH)                                                                                         \
    hipLaunchKernelGGL((k_reduce_update<GT, HH>), dim3(grid), dim3(kThreads), 0, s, c->d_span_first,       \
                       c->d_tile_prefix, c->d_numel, d_ptrs, c->d_partials, c->d_book, c->d_lr, sa, c->n_tiles, \
                       c->span_tiles, c->n_spans, S, row_len, inv_S, rho, lambda)
    if (S >= 16) LAUNCH(8);
    else if (S >= 8) LAUNCH(4);
    else if (S >= 4) LAUNCH(2);
    else LAUNCH(1);
#undef LAUNCH
}


// ADASCALE_LAGGED_R on the fused step.  eta_t is known before any gradient is read, so the grid
// barrier is not needed for the result, and the instances without it (k_scalars behind them)
// save its 2.5 us: 15.3 against 17.7 us at d = 1 M, S = 4.  But the barrier also keeps phase 2's
// writes of the early workgroups out of the late workgroups' gradient sweep, and on anything
// larger that is worth more: with the barrier 87.6 against 92.6 us at d = 11 M, S = 8, 312.7
// against 317-324 us at d = 25.6 M, S = 16, 7.58 against 7.71 ms at d = 351 M, S = 64 bf16 (one
// session; the barrier kernel evaluates the same prior-iteration gain itself).  The instances
// without barrier are taken while a workgroup's share of the step is estimated below 50 us.
bool lag_barrier_free(const adascale_ctx *c, int S)
{
    if (!(c->cfg.flags & ADASCALE_LAGGED_R)) return false;
    const double b = c->cfg.grad_dtype == ADASCALE_F32 ? 4.0 : 2.0;
    const double us = (double)c->f_tpb * kFTile * (S * b + 16.0) / 27.0e3;  // 27 GB/s per workgroup at 6.9 TB/s
    return us < 50.0;
}

}  // namespace

// ---------------------------------------------------------------------------------------------
extern "C" {

const char *adascale_last_error(const adascale_ctx *ctx) { return ctx ? ctx->err : g_init_error; }

int64_t adascale_step_bytes(const adascale_ctx *c)
{
    if (!c) return 0;
    const int64_t b = c->cfg.grad_dtype == ADASCALE_F32 ? 4 : 2;
    return (int64_t)c->cfg.S * c->d * b + (c->cfg.weight_decay != 0.0 ? 24 : 20) * c->d;
}

int adascale_step_path(const adascale_ctx *c)
{
    if (!c) return ADASCALE_PATH_GENERAL;
    if (c->fused_ok && fused_kernel_for(c->cfg.grad_dtype, c->cfg.S, c->f_level, lag_barrier_free(c, c->cfg.S)))
        return ADASCALE_PATH_FUSED;
    if (c->stream_ok && stream_kernel_for(c->cfg.grad_dtype, c->cfg.S)) return ADASCALE_PATH_STREAMING;
    return ADASCALE_PATH_GENERAL;
}

int adascale_kernel_shape(int32_t grad_dtype, int32_t S, int32_t shape[3])
{
    int hg = 0, nh = 0;
    if ((grad_dtype != ADASCALE_F32 && grad_dtype != ADASCALE_BF16) || !shape || !fused_shape(grad_dtype, S, &hg, &nh))
        return 0;
    shape[0] = hg;
    shape[1] = nh;
    shape[2] = padded_scale(grad_dtype, S);
    bool fused = true;
    for (int level = 0; level < kFRegLevels; ++level)
        for (int lag = 0; lag < 2; ++lag) fused = fused && fused_kernel_for(grad_dtype, S, level, lag != 0) != nullptr;
    return (fused ? 1 : 0) | (stream_kernel_for(grad_dtype, S) ? 2 : 0);
}

int adascale_plan(const adascale_config *cfg, const adascale_tuning *tuning, int32_t compute_units, int64_t lds_bytes,
                  adascale_plan_info *out)
{
    const adascale_tuning tun = tuning ? *tuning : adascale_tuning{};
    if (!cfg || !out || cfg->S < 1 || cfg->n_tensors < 0 || (cfg->n_tensors > 0 && !cfg->numel) || compute_units < 1 ||
        lds_bytes < 0 || (cfg->grad_dtype != ADASCALE_F32 && cfg->grad_dtype != ADASCALE_BF16))
        return fail(nullptr, ADASCALE_EINVAL, "bad argument to adascale_plan");
    for (int k = 0; k < cfg->n_tensors; ++k)
        if (cfg->numel[k] < 0) return fail(nullptr, ADASCALE_EINVAL, "negative numel");
    *out = adascale_plan_info{};
    std::vector<long long> numel(cfg->numel, cfg->numel + cfg->n_tensors);
    long long d = 0;
    for (long long n : numel) d += n;
    long long full = 0, ragged = 0;
    const bool tiles_ok = d > 0 && plan_tiles(numel.data(), cfg->n_tensors, &full, &ragged);
    out->path = ADASCALE_PATH_GENERAL;
    if (!tiles_ok) return ADASCALE_OK;
    out->full_tiles = full;
    out->ragged_tiles = ragged;
    const bool stream_ok = plan_stream_ok(tun, (size_t)lds_bytes);
    if (stream_ok) out->stream_grid = plan_stream_grid(full, ragged, compute_units);
    const FusedPlan f = plan_fused(tun, full, ragged, compute_units, (size_t)lds_bytes, stream_ok);
    const bool lag = (cfg->flags & ADASCALE_LAGGED_R) != 0;
    if (f.ok) {
        out->fused_grid = f.grid;
        out->tiles_per_workgroup = f.tpb;
        out->register_tiles = fused_regs_at(f.level);
        out->lds_tiles = std::max(0, std::min(f.tpb - fused_regs_at(f.level), f.lds_cap));
        out->on_chip_percent = f.on_chip_pct;
    }
    if (f.ok && fused_kernel_for(cfg->grad_dtype, cfg->S, f.level, lag)) out->path = ADASCALE_PATH_FUSED;
    else if (stream_ok && stream_kernel_for(cfg->grad_dtype, cfg->S)) out->path = ADASCALE_PATH_STREAMING;
    return ADASCALE_OK;
}

int adascale_uses_fused_step(const adascale_ctx *c) { return adascale_step_path(c) == ADASCALE_PATH_FUSED ? 1 : 0; }

int adascale_fail_next_barrier(adascale_ctx *c)
{
    if (!c) return ADASCALE_EINVAL;
    if (adascale_step_path(c) != ADASCALE_PATH_FUSED || lag_barrier_free(c, c->cfg.S))
        return fail(c, ADASCALE_ESTATE, "the next step has no grid barrier");
    c->fail_next = true;
    return ADASCALE_OK;
}

int64_t adascale_step_moved_bytes(const adascale_ctx *c)
{
    if (!c) return 0;
    const int64_t b = c->cfg.grad_dtype == ADASCALE_F32 ? 4 : 2;
    const bool decay = c->cfg.weight_decay != 0.0, lag = (c->cfg.flags & ADASCALE_LAGGED_R) != 0;
    const int64_t grads = (int64_t)c->cfg.S * c->d * b;
    const int path = adascale_step_path(c);
    if (path == ADASCALE_PATH_GENERAL) return grads + (lag ? 16 : 24) * c->d;  // one sweep / mean gradient out and in
    int64_t ragged = 0;  // elements in ragged last tiles
    for (const FTile &t : c->ctiles) ragged += c->numel[t.k] - (int64_t)t.local * kFTile;
    const int64_t full = (int64_t)c->ftiles.size() * kFTile;
    const int64_t in_sweep = decay ? 24 : 20;  // v read and written (w read) in the sweep; w, v read and w written after it
    if (path == ADASCALE_PATH_STREAMING) {
        if (!c->stream_momentum) return grads + 24 * c->d;
        // ragged tiles: mean gradient out and in, then w, v read and v written, then the update pass
        return grads + in_sweep * full + 32 * ragged;
    }
    // fused: workgroup b holds full tiles b, b + G, ...; the first q_hbm of them stay on chip
    int regs = 0;
    (void)fused_kernel_for(c->cfg.grad_dtype, c->cfg.S, c->f_level, lag_barrier_free(c, c->cfg.S), &regs);
    const int q_hbm = std::min(regs + std::max(0, std::min(c->f_tpb - regs, c->f_lds_cap)), c->f_tpb);
    const int64_t nt = (int64_t)c->ftiles.size();
    int64_t on_chip = 0;
    for (int g = 0; g < c->f_grid; ++g) {
        const int64_t n_valid = g < nt ? (nt - 1 - g) / c->f_grid + 1 : 0;
        on_chip += std::min<int64_t>(n_valid, q_hbm);
    }
    return grads + 16 * on_chip * kFTile + in_sweep * (nt - on_chip) * kFTile + 24 * ragged;
}

int adascale_init(const adascale_config *cfg, adascale_ctx **out) { return adascale_init_tuned(cfg, nullptr, out); }

int adascale_init_tuned(const adascale_config *cfg, const adascale_tuning *tuning, adascale_ctx **out)
{
    if (out) *out = nullptr;
    if (!cfg || !out) return fail(nullptr, ADASCALE_EINVAL, "null cfg or out");
    if (cfg->S < 1) return fail(nullptr, ADASCALE_EINVAL, "S must be >= 1");
    if (cfg->n_tensors < 0 || (cfg->n_tensors > 0 && !cfg->numel))
        return fail(nullptr, ADASCALE_EINVAL, "bad tensor list");
    if (cfg->grad_dtype != ADASCALE_F32 && cfg->grad_dtype != ADASCALE_BF16)
        return fail(nullptr, ADASCALE_EINVAL, "unknown gradient dtype");
    if (!(cfg->momentum >= 0.0 && cfg->momentum < 1.0)) return fail(nullptr, ADASCALE_EINVAL, "momentum outside [0,1)");
    if (!(cfg->weight_decay >= 0.0)) return fail(nullptr, ADASCALE_EINVAL, "negative weight decay");
    if (!(cfg->theta < 1.0)) return fail(nullptr, ADASCALE_EINVAL, "theta must be < 1");
    if (!cfg->lr_table || cfg->lr_table_len < 1) return fail(nullptr, ADASCALE_EINVAL, "empty lr table");
    if (cfg->flags & ~(ADASCALE_LAGGED_R | ADASCALE_EST_NORM_RATIO | ADASCALE_NO_POINTER_CHECK |
                       ADASCALE_COOPERATIVE_LAUNCH))
        return fail(nullptr, ADASCALE_EINVAL, "unknown flag bits");
    for (int k = 0; k < cfg->n_tensors; ++k)
        if (cfg->numel[k] < 0) return fail(nullptr, ADASCALE_EINVAL, "negative numel");
    if (tuning && (tuning->force_path < ADASCALE_FORCE_NONE || tuning->force_path > ADASCALE_FORCE_STREAMING ||
                   tuning->fused_max_grid < 0 || tuning->fused_min_percent < 0 || tuning->fused_min_percent > 100 ||
                   tuning->barrier_spin_limit < 0 || (tuning->stream_via_scratch != 0 && tuning->stream_via_scratch != 1)))
        return fail(nullptr, ADASCALE_EINVAL, "bad tuning record");

    adascale_ctx *c = new (std::nothrow) adascale_ctx();
    if (!c) return fail(nullptr, ADASCALE_ENOMEM, "host allocation failed");
    c->cfg = *cfg;
    c->cfg.numel = nullptr;
    c->cfg.lr_table = nullptr;
    if (c->cfg.theta < 0.0) c->cfg.theta = std::max(1.0 - cfg->S / 1000.0, 0.0);
    if (c->cfg.eps <= 0.0) c->cfg.eps = 1e-6;
    c->vec = cfg->grad_dtype == ADASCALE_F32 ? 4 : 8;
    c->tile = kThreads * c->vec;
    if (tuning) c->tun = *tuning;

    const int N = cfg->n_tensors;
    c->numel.assign(cfg->numel, cfg->numel + N);
    c->tile_prefix.assign(N + 1, 0);
    c->gbar_off.assign(N, 0);
    size_t goff = 0;
    long long tiles = 0;
    for (int k = 0; k < N; ++k) {
        c->d += c->numel[k];
        tiles += (c->numel[k] + c->tile - 1) / c->tile;
        if (tiles > 0x7fffff00LL) {
            delete c;
            return fail(nullptr, ADASCALE_EINVAL, "parameter list too large");
        }
        c->tile_prefix[k + 1] = (int)tiles;
        c->gbar_off[k] = goff;
        goff += ((size_t)c->numel[k] + 63) / 64 * 64;  // 256-byte aligned starts
    }
    c->gbar_len = std::max<size_t>(goff, 64);
    c->n_tiles = (int)tiles;
    c->n_spans = (c->n_tiles + c->span_tiles - 1) / c->span_tiles;
    c->span_first.assign(std::max(c->n_spans, 1), 0);
    for (int s = 0, k = 0; s < c->n_spans; ++s) {
        const int t = s * c->span_tiles;
        while (t >= c->tile_prefix[k + 1]) ++k;
        c->span_first[s] = k;
    }

    int rc = ADASCALE_OK;
    DeviceGuard guard;
    auto body = [&]() -> int {
        int ndev = 0;
        HIP_TRY(c, hipGetDeviceCount(&ndev));
        if (cfg->device < 0 || cfg->device >= ndev) return fail(c, ADASCALE_EINVAL, "no such device");
        HIP_TRY(c, guard.enter(cfg->device));
        HIP_TRY(c, hipMalloc(&c->d_span_first, sizeof(int) * c->span_first.size()));
        HIP_TRY(c, hipMalloc(&c->d_tile_prefix, sizeof(int) * (N + 1)));
        HIP_TRY(c, hipMalloc(&c->d_numel, sizeof(long long) * std::max(N, 1)));
        HIP_TRY(c, hipMalloc(&c->d_lr, sizeof(float) * cfg->lr_table_len));
        // partial slots: one per span (reduce kernel), per workgroup (fused step), or per workgroup
        // plus one per pair of 512-lane tiles (streaming reduce kernel)
        const size_t n_slots = std::max<size_t>((size_t)c->n_spans, (size_t)kFMaxGrid + (size_t)(c->d / (2 * kFTile)) + 1);
        HIP_TRY(c, hipMalloc(&c->d_partials, sizeof(double) * 2 * n_slots));
        HIP_TRY(c, hipMalloc(&c->d_book, sizeof(DevBook)));
        HIP_TRY(c, hipMemset(c->d_book, 0, sizeof(DevBook)));
        HIP_TRY(c, hipHostMalloc(&c->h_book, sizeof(DevBook), hipHostMallocDefault));
        for (int j = 0; j < kTables; ++j) HIP_TRY(c, hipEventCreateWithFlags(&c->tab_ev[j], hipEventDisableTiming));
        HIP_TRY(c, hipMemcpy(c->d_span_first, c->span_first.data(), sizeof(int) * c->span_first.size(),
                             hipMemcpyHostToDevice));
        HIP_TRY(c, hipMemcpy(c->d_tile_prefix, c->tile_prefix.data(), sizeof(int) * (N + 1), hipMemcpyHostToDevice));
        if (N > 0)
            HIP_TRY(c, hipMemcpy(c->d_numel, c->numel.data(), sizeof(long long) * N, hipMemcpyHostToDevice));
        HIP_TRY(c, hipMemcpy(c->d_lr, cfg->lr_table, sizeof(float) * cfg->lr_table_len, hipMemcpyHostToDevice));
        HIP_TRY(c, hipMemset(c->d_partials, 0, sizeof(double) * 2 * n_slots));
        const int trc = setup_tiles(c);
        if (trc != ADASCALE_OK) return trc;
        const int frc = setup_fused(c);
        if (frc != ADASCALE_OK) return frc;
        return alloc_pointer_tables(c, cfg->S);
    };
    rc = body();
    if (rc != ADASCALE_OK) {
        snprintf(g_init_error, sizeof g_init_error, "%s", c->err);
        adascale_destroy(c);
        return rc;
    }
    *out = c;
    return ADASCALE_OK;
}

void adascale_destroy(adascale_ctx *c)
{
    if (!c) return;
    DeviceGuard guard;
    (void)guard.enter(c->cfg.device);
    (void)hipDeviceSynchronize();
    (void)hipFree(c->d_span_first);
    (void)hipFree(c->d_tile_prefix);
    (void)hipFree(c->d_numel);
    (void)hipFree(c->d_gbar);
    (void)hipFree(c->d_cold_gbar);
    (void)hipFree(c->d_lr);
    (void)hipFree(c->d_partials);
    (void)hipFree(c->d_book);
    (void)hipFree(c->d_ftiles);
    (void)hipFree(c->d_ctiles);
    if (c->h_book) (void)hipHostFree(c->h_book);
    for (int j = 0; j < kTables; ++j) {
        (void)hipFree(c->d_tab[j]);
        if (c->h_tab[j]) (void)hipHostFree(c->h_tab[j]);
        if (c->tab_ev[j]) (void)hipEventDestroy(c->tab_ev[j]);
    }
    for (hipEvent_t e : c->prof_ev) (void)hipEventDestroy(e);
    delete c;
}

int adascale_set_scale(adascale_ctx *c, int32_t S_new, double theta)
{
    if (!c) return ADASCALE_EINVAL;
    if (S_new < 1) return fail(c, ADASCALE_EINVAL, "S must be >= 1");
    if (!(theta < 1.0)) return fail(c, ADASCALE_EINVAL, "theta must be < 1");
    DeviceGuard guard;
    HIP_TRY(c, guard.enter(c->cfg.device));
    const int rc = alloc_pointer_tables(c, S_new);
    if (rc != ADASCALE_OK) return rc;
    c->cfg.S = S_new;
    c->cfg.theta = theta < 0.0 ? std::max(1.0 - S_new / 1000.0, 0.0) : theta;
    forget_tables(c);  // their rows have the old scale's length
    return ADASCALE_OK;
}

int adascale_set_state(adascale_ctx *c, int64_t step, double tau, double sigma2_bar, double mu2_bar, void *hip_stream)
{
    if (!c) return ADASCALE_EINVAL;
    if (step < 0 || !(tau >= 0.0) || !(sigma2_bar >= 0.0) || !(mu2_bar >= 0.0))
        return fail(c, ADASCALE_EINVAL, "state values must be non-negative");
    DeviceGuard guard;
    HIP_TRY(c, guard.enter(c->cfg.device));
    hipLaunchKernelGGL(k_set_state, dim3(1), dim3(64), 0, (hipStream_t)hip_stream, c->d_book, (long long)step, tau,
                       sigma2_bar, mu2_bar, (long long)c->cfg.lr_table_len);
    HIP_TRY(c, hipGetLastError());
    c->failed = false;
    return ADASCALE_OK;
}

int adascale_get_state(adascale_ctx *c, adascale_state *out, void *hip_stream)
{
    if (!c) return ADASCALE_EINVAL;
    if (!out) return fail(c, ADASCALE_EINVAL, "null out");
    hipStream_t s = (hipStream_t)hip_stream;
    DeviceGuard guard;
    HIP_TRY(c, guard.enter(c->cfg.device));
    HIP_TRY(c, hipMemcpyAsync(c->h_book, c->d_book, sizeof(DevBook), hipMemcpyDeviceToHost, s));
    HIP_TRY(c, hipStreamSynchronize(s));
    if (c->h_book->fault) {
        c->failed = true;
        return fail(c, ADASCALE_ESTATE, "a fused step gave up waiting at its grid barrier: w, v and the state are invalid; "
                                        "restore them and call adascale_set_state");
    }
    const DevState &h = c->h_book->st[c->h_book->epoch & 1];
    out->step = h.step;
    out->tau = h.tau;
    out->r = h.r;
    out->lr_eff = h.lr_eff;
    out->sum_sq = h.A;
    out->sq_mean = h.B;
    out->sigma2_hat = h.sig_hat;
    out->mu2_hat = h.mu_hat;
    out->sigma2_bar = h.sig_bar;
    out->mu2_bar = h.mu_bar;
    out->done = h.done;
    return ADASCALE_OK;
}

int adascale_step(adascale_ctx *c, void *const *w, void *const *mom, const void *const *grads, void *hip_stream)
{
    if (!c) return ADASCALE_EINVAL;
    const int N = (int)c->numel.size();
    const int S = c->cfg.S;
    if (N > 0 && (!w || !mom || !grads)) return fail(c, ADASCALE_EINVAL, "null pointer array");
    hipStream_t s = (hipStream_t)hip_stream;
    DeviceGuard guard;
    HIP_TRY(c, guard.enter(c->cfg.device));

    if (c->failed)
        return fail(c, ADASCALE_ESTATE, "an earlier step failed at its grid barrier; restore w, v and call adascale_set_state");
    // Is the stream being captured into a graph?  Then nothing here may wait, copy or allocate, and
    // what is launched must stay valid for every replay.
    hipStreamCaptureStatus cap_status = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(s, &cap_status) != hipSuccess) {
        (void)hipGetLastError();
        cap_status = hipStreamCaptureStatusNone;
    }
    const bool capturing = cap_status != hipStreamCaptureStatusNone;

    // the general kernels pass the whole mean gradient through memory
    const int path = adascale_step_path(c);
    if (!c->d_gbar && (path == ADASCALE_PATH_GENERAL || (path == ADASCALE_PATH_STREAMING && !c->stream_momentum))) {
        if (capturing)
            return fail(c, ADASCALE_ESTATE, "the first step on the general kernels allocates: run one step outside the capture first");
        HIP_TRY(c, hipMalloc(&c->d_gbar, sizeof(float) * c->gbar_len));
        forget_tables(c);  // they point at the ragged-tile scratch
    }

    // The device pointer table [N][3 + S'] of this call.  The device keeps the tables of the last
    // kTables distinct pointer sets, so a caller that alternates between a few sets of buffers
    // uploads nothing; a new set replaces the one used longest ago.
    const int S_pad = padded_scale(c->cfg.grad_dtype, S);
    const int row_len = S_pad + kRowG;
    const size_t len = table_len(c, S);
    const unsigned long long *d_ptrs = c->d_tab[0];
    c->steps_issued += 1;
    if (len > 0) {
        c->tab_build.resize(len);
        unsigned long long *tab = c->tab_build.data();
        for (int k = 0; k < N; ++k) {
            unsigned long long *row = tab + (size_t)k * row_len;
            row[kRowW] = (unsigned long long)(uintptr_t)w[k];
            row[kRowV] = (unsigned long long)(uintptr_t)mom[k];
            row[kRowGbar] = c->d_gbar ? (unsigned long long)(uintptr_t)(c->d_gbar + c->gbar_off[k]) : c->cold_base[k];
            for (int i = 0; i < S_pad; ++i)
                row[kRowG + i] = (unsigned long long)(uintptr_t)grads[(size_t)std::min(i, S - 1) * N + k];
        }
        int slot = -1;
        for (int i = 0; i < kTables && slot < 0; ++i) {  // the table of the last step first
            const int j = (c->tab_last + i) % kTables;
            if (c->tab_len[j] == len && memcmp(c->h_tab[j], tab, len * sizeof(unsigned long long)) == 0) slot = j;
        }
        if (slot < 0 && capturing)
            return fail(c, ADASCALE_ESTATE, "this set of tensor pointers has no table on the device yet: run one step with it "
                                            "outside the capture first");
        if (slot < 0) {
            const size_t gb = c->cfg.grad_dtype == ADASCALE_F32 ? 4 : 2;
            uintptr_t lo = 1, hi = 0;
            for (int k = 0; k < N; ++k) {
                if (c->numel[k] == 0) continue;
                const unsigned long long *row = tab + (size_t)k * row_len;
                for (int j = 0; j < row_len; ++j) {
                    if (j == kRowGbar) continue;
                    if (!row[j]) return fail(c, ADASCALE_EINVAL, "null tensor pointer (tensor %d, slot %d)", k, j);
                    const size_t eb = j < kRowG ? 4 : gb;
                    if (row[j] % eb) return fail(c, ADASCALE_EINVAL, "misaligned tensor pointer (tensor %d, slot %d)", k, j);
                    if (!(c->cfg.flags & ADASCALE_NO_POINTER_CHECK) &&
                        !device_range_ok((const void *)(uintptr_t)row[j], (size_t)c->numel[k] * eb, c->cfg.device, lo, hi))
                        return fail(c, ADASCALE_EINVAL, "tensor %d, slot %d: not device memory of %lld elements", k, j,
                                    c->numel[k]);
                }
            }
            slot = -1;  // an empty table if there is one, else the one used longest ago; never one a graph refers to
            for (int j = 0; j < kTables && (slot < 0 || c->tab_len[slot] != 0); ++j) {
                if (c->tab_captured[j]) continue;
                if (slot < 0 || c->tab_len[j] == 0 || c->tab_used[j] < c->tab_used[slot]) slot = j;
            }
            if (slot < 0) return fail(c, ADASCALE_ESTATE, "every pointer table of this context is held by a captured step");
            // the mirror is the staging buffer: its last upload must have left it (long ago, normally)
            if (c->tab_uploaded[slot]) HIP_TRY(c, hipEventSynchronize(c->tab_ev[slot]));
            c->tab_len[slot] = 0;
            memcpy(c->h_tab[slot], tab, len * sizeof(unsigned long long));
            // stream order puts the copy behind every earlier kernel that reads this table
            HIP_TRY(c, hipMemcpyAsync(c->d_tab[slot], c->h_tab[slot], len * sizeof(unsigned long long), hipMemcpyHostToDevice, s));
            HIP_TRY(c, hipEventRecord(c->tab_ev[slot], s));
            c->tab_uploaded[slot] = true;
            c->tab_len[slot] = len;
        }
        c->tab_used[slot] = c->steps_issued;
        c->tab_last = slot;
        if (capturing) c->tab_captured[slot] = true;
        d_ptrs = c->d_tab[slot];
    }

    hipEvent_t *pe = nullptr;
    if (c->prof_on && c->prof_n < c->prof_cap && !capturing) pe = &c->prof_ev[(size_t)4 * c->prof_n++];
    if (pe) HIP_TRY(c, hipEventRecord(pe[0], s));
    ScalarArgs sa{S, c->cfg.flags, c->cfg.theta, c->cfg.eps, (long long)c->cfg.lr_table_len};
    const bool lag = (c->cfg.flags & ADASCALE_LAGGED_R) != 0;
    int f_regs = 0;
    const bool lag_kernel = lag_barrier_free(c, S);
    const void *fused_fn = c->fused_ok ? fused_kernel_for(c->cfg.grad_dtype, S, c->f_level, lag_kernel, &f_regs) : nullptr;
    const int f_lds_tiles = std::max(0, std::min(c->f_tpb - f_regs, c->f_lds_cap));
    if (fused_fn) {
        FusedArgs fa{};
        fa.tiles = c->d_ftiles;
        fa.cold = c->d_ctiles;
        fa.n_cold = (int)c->ctiles.size();
        fa.numel = c->d_numel;
        fa.ptrs = d_ptrs;
        fa.partials = c->d_partials;
        fa.book = c->d_book;
        fa.lr = c->d_lr;
        fa.barrier_extra = c->fail_next && !lag_kernel ? 1 : 0;  // adascale_fail_next_barrier: an arrival that never comes
        c->fail_next = false;
        fa.spin_limit = c->tun.barrier_spin_limit > 0 ? c->tun.barrier_spin_limit : kFSpinLimit;
        fa.n_tiles = (int)c->ftiles.size();
        fa.tiles_per_block = c->f_tpb;
        fa.lds_tiles = f_lds_tiles;
        fa.S = S;
        fa.row_len = row_len;
        int f_hg = 0;
        (void)fused_shape(c->cfg.grad_dtype, S, &f_hg, &fa.nh);
        fa.inv_S = 1.0 / (double)S;
        fa.rho = (float)c->cfg.momentum;
        fa.lambda = (float)c->cfg.weight_decay;
        fa.win_inv = burst_window_factor(c, S, c->f_grid, std::min(f_lds_tiles, kBurstMax), 16.0);
        fa.sc = sa;
        void *args[] = {&fa};
        const size_t lds_bytes = (size_t)f_lds_tiles * kFThreads * sizeof(f4);
        if (c->cfg.flags & ADASCALE_COOPERATIVE_LAUNCH) {
            HIP_TRY(c, hipLaunchCooperativeKernel(fused_fn, dim3(c->f_grid), dim3(kFThreads), args, lds_bytes, s));
        } else if (capturing) {
            // a replay is ordered by the graph's own dependencies; keeping it apart from fused steps
            // on other streams is then the caller's business
            HIP_TRY(c, hipLaunchKernel(fused_fn, dim3(c->f_grid), dim3(kFThreads), args, lds_bytes, s));
        } else {
            // Ordinary launch (a cooperative one costs ~15 us more per step here).  The grid is one
            // workgroup per CU, so all of it becomes resident as soon as the CUs are free; what
            // must not happen is two fused kernels each holding part of the chip and waiting for
            // the rest.  Fused launches of this process on one device are therefore chained: a
            // launch on another stream than the previous one first waits for that one's event.
            FusedChain &ch = g_chain[c->cfg.device % kMaxDevices];
            std::lock_guard<std::mutex> lock(ch.m);
            if (!ch.ev) HIP_TRY(c, hipEventCreateWithFlags(&ch.ev, hipEventDisableTiming));
            if (ch.used && ch.last_stream != s) HIP_TRY(c, hipStreamWaitEvent(s, ch.ev, 0));
            HIP_TRY(c, hipLaunchKernel(fused_fn, dim3(c->f_grid), dim3(kFThreads), args, lds_bytes, s));
            HIP_TRY(c, hipEventRecord(ch.ev, s));
            ch.used = true;
            ch.last_stream = s;
        }
        if (pe) HIP_TRY(c, hipEventRecord(pe[1], s));
        if (lag_kernel) {
            hipLaunchKernelGGL(k_scalars, dim3(1), dim3(kScalarThreads), 0, s, c->d_partials, c->f_grid, c->d_book, c->d_lr,
                               sa);
            HIP_TRY(c, hipGetLastError());
        }
        if (pe)
            for (int j = 2; j < 4; ++j) HIP_TRY(c, hipEventRecord(pe[j], s));
        return ADASCALE_OK;
    }
    const int grid = c->n_spans;
    const void *stream_fn = c->stream_ok ? stream_kernel_for(c->cfg.grad_dtype, S) : nullptr;
    int n_partials = c->n_spans;
    if (stream_fn) {
        StreamArgs ra{};
        ra.tiles = c->d_ftiles;
        ra.cold = c->d_ctiles;
        ra.numel = c->d_numel;
        ra.ptrs = d_ptrs;
        ra.partials = c->d_partials;
        ra.claim = &c->d_book->claim;
        ra.n_tiles = (int)c->ftiles.size();
        ra.n_cold = (int)c->ctiles.size();
        ra.S = S;
        ra.row_len = row_len;
        int hg = 0;
        (void)fused_shape(c->cfg.grad_dtype, S, &hg, &ra.nh);
        ra.momentum = c->stream_momentum ? 1 : 0;
        ra.rho = (float)c->cfg.momentum;
        ra.lambda = (float)c->cfg.weight_decay;
        ra.inv_S = 1.0 / (double)S;
        ra.keep = c->s_keep;
        ra.win_inv = burst_window_factor(c, S, c->s_grid, c->s_keep, 32.0);
        if (ra.win_inv == 0) ra.keep = 0;
        void *args[] = {&ra};
        HIP_TRY(c, hipLaunchKernel(stream_fn, dim3(c->s_grid), dim3(kFThreads), args, c->s_lds, s));
        n_partials = c->s_grid + (ra.n_tiles + 1) / 2;
    }
    // Prior-iteration gain without the streaming kernel: single pass (reduce + update), then the
    // scalars.  With it the order is the general one below: k_scalars derives eta_t from the prior
    // averages and k_update applies it.
    if (lag && !stream_fn) {
        if (grid > 0) {
            if (c->cfg.grad_dtype == ADASCALE_F32) launch_reduce_update<float>(c, d_ptrs, grid, s, S, sa);
            else launch_reduce_update<Bf16>(c, d_ptrs, grid, s, S, sa);
            HIP_TRY(c, hipGetLastError());
        }
        if (pe) HIP_TRY(c, hipEventRecord(pe[1], s));
        hipLaunchKernelGGL(k_scalars, dim3(1), dim3(kScalarThreads), 0, s, c->d_partials, n_partials, c->d_book, c->d_lr, sa);
        HIP_TRY(c, hipGetLastError());
        if (pe)
            for (int j = 2; j < 4; ++j) HIP_TRY(c, hipEventRecord(pe[j], s));
        return ADASCALE_OK;
    }
    if (!stream_fn && grid > 0) {
        if (c->cfg.grad_dtype == ADASCALE_F32) launch_reduce<float>(c, d_ptrs, grid, s, S);
        else launch_reduce<Bf16>(c, d_ptrs, grid, s, S);
        HIP_TRY(c, hipGetLastError());
    }
    if (pe) HIP_TRY(c, hipEventRecord(pe[1], s));
    hipLaunchKernelGGL(k_scalars, dim3(1), dim3(kScalarThreads), 0, s, c->d_partials, n_partials, c->d_book, c->d_lr, sa);
    HIP_TRY(c, hipGetLastError());
    if (pe) HIP_TRY(c, hipEventRecord(pe[2], s));
    if (grid > 0) {
        const float rho = (float)c->cfg.momentum, lambda = (float)c->cfg.weight_decay;
#define LAUNCH(VV)                                                                                       \
    hipLaunchKernelGGL((k_update<VV>), dim3(grid), dim3(kThreads), 0, s, c->d_span_first, c->d_tile_prefix, \
                       c->d_numel, d_ptrs, c->d_book, c->n_tiles, c->span_tiles, c->n_spans, row_len, rho,  \
                       lambda)
        if (stream_fn && c->stream_momentum) {
            ApplyArgs aa{c->d_ftiles, c->d_ctiles, c->d_numel, d_ptrs, c->d_book, (int)c->ftiles.size(),
                         (int)c->ctiles.size(), row_len};
            hipLaunchKernelGGL(k_apply, dim3(c->s_grid), dim3(kFThreads), 0, s, aa);
        } else {
            if (c->vec == 4) LAUNCH(4);
            else LAUNCH(8);
        }
#undef LAUNCH
        HIP_TRY(c, hipGetLastError());
    }
    if (pe) HIP_TRY(c, hipEventRecord(pe[3], s));
    return ADASCALE_OK;
}

// Address of this device's copy of `scratch` (the device must be current).
static hipError_t flat_scratch_on(int device, FlatScratch **out)
{
    std::lock_guard<std::mutex> lock(g_flat_mutex);
    if (!g_flat_scratch[device]) {
        void *p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        g_flat_scratch[device] = static_cast<FlatScratch *>(p);
    }
    *out = g_flat_scratch[device];
    return hipSuccess;
}

int adascale_step_flat(const adascale_flat_step *a, void *hip_stream)
{
    if (!a) return fail(nullptr, ADASCALE_EINVAL, "null argument record");
    if (a->S < 1 || a->S > kFlatMaxScale)
        return fail(nullptr, ADASCALE_EINVAL, "adascale_step_flat takes 1 to %d gradient buffers, got %d", kFlatMaxScale, a->S);
    if (a->numel < 0 || a->numel > ADASCALE_FLAT_MAX_NUMEL)
        return fail(nullptr, ADASCALE_EINVAL, "adascale_step_flat takes at most %lld elements", (long long)ADASCALE_FLAT_MAX_NUMEL);
    if (a->grad_dtype != ADASCALE_F32 && a->grad_dtype != ADASCALE_BF16)
        return fail(nullptr, ADASCALE_EINVAL, "unknown gradient dtype");
    if (!(a->momentum >= 0.0 && a->momentum < 1.0)) return fail(nullptr, ADASCALE_EINVAL, "momentum outside [0,1)");
    if (!(a->weight_decay >= 0.0)) return fail(nullptr, ADASCALE_EINVAL, "negative weight decay");
    if (!(a->theta < 1.0)) return fail(nullptr, ADASCALE_EINVAL, "theta must be < 1");
    if (!a->lr_table || a->lr_table_len < 1) return fail(nullptr, ADASCALE_EINVAL, "empty lr table");
    if (a->flags & ~(ADASCALE_LAGGED_R | ADASCALE_EST_NORM_RATIO | ADASCALE_NO_POINTER_CHECK))
        return fail(nullptr, ADASCALE_EINVAL, "flag not supported by adascale_step_flat");
    if (!a->state || (uintptr_t)a->state % 8) return fail(nullptr, ADASCALE_EINVAL, "null or misaligned state record");
    if (a->device < 0 || a->device >= kMaxDevices) return fail(nullptr, ADASCALE_EINVAL, "no such device");
    const size_t gb = a->grad_dtype == ADASCALE_F32 ? 4 : 2;
    FlatPointers fp{};
    if (a->numel > 0) {
        if (!a->w || !a->mom || !a->grads) return fail(nullptr, ADASCALE_EINVAL, "null tensor pointer");
        if ((uintptr_t)a->w % 4 || (uintptr_t)a->mom % 4) return fail(nullptr, ADASCALE_EINVAL, "misaligned tensor pointer");
        fp.w = (unsigned long long)(uintptr_t)a->w;
        fp.v = (unsigned long long)(uintptr_t)a->mom;
        for (int i = 0; i < a->S; ++i) {
            if (!a->grads[i] || (uintptr_t)a->grads[i] % gb)
                return fail(nullptr, ADASCALE_EINVAL, "null or misaligned gradient pointer (buffer %d)", i);
            fp.g[i] = (unsigned long long)(uintptr_t)a->grads[i];
        }
    }
    hipStream_t s = (hipStream_t)hip_stream;
    DeviceGuard guard;
    HIP_TRY(nullptr, guard.enter(a->device));
    if (a->numel > 0 && !(a->flags & ADASCALE_NO_POINTER_CHECK)) {
        uintptr_t lo = 1, hi = 0;
        bool ok = device_range_ok(a->w, (size_t)a->numel * 4, a->device, lo, hi) &&
                  device_range_ok(a->mom, (size_t)a->numel * 4, a->device, lo, hi);
        for (int i = 0; i < a->S && ok; ++i) ok = device_range_ok(a->grads[i], (size_t)a->numel * gb, a->device, lo, hi);
        if (!ok) return fail(nullptr, ADASCALE_EINVAL, "a tensor pointer is not device memory of %lld elements", (long long)a->numel);
    }
    FlatScratch *sc = nullptr;
    HIP_TRY(nullptr, flat_scratch_on(a->device, &sc));

    const int vec = a->grad_dtype == ADASCALE_F32 ? 4 : 8;
    const long long tile = (long long)kThreads * vec;
    const int n_tiles = (int)((a->numel + tile - 1) / tile);
    const int grid = std::max(1, std::min(n_tiles, kFlatMaxGrid));
    const double theta = a->theta < 0.0 ? std::max(1.0 - a->S / 1000.0, 0.0) : a->theta;
    const ScalarArgs sa{a->S, a->flags, theta, a->eps <= 0.0 ? 1e-6 : a->eps, (long long)a->lr_table_len};
    const double inv_S = 1.0 / (double)a->S;
    const float rho = (float)a->momentum, lambda = (float)a->weight_decay;
    adascale_state *user = static_cast<adascale_state *>(a->state);

    hipLaunchKernelGGL(k_flat_setup, dim3(1), dim3(kFlatMaxScale), 0, s, sc, fp, a->S, user);
#define LAUNCH(GT, HH) hipLaunchKernelGGL((k_flat_sweep<GT, HH>), dim3(grid), dim3(kThreads), 0, s, sc, (long long)a->numel, n_tiles, a->S, inv_S, rho, lambda)
    if (a->grad_dtype == ADASCALE_F32) {
        if (a->S >= 16) LAUNCH(float, 8);
        else if (a->S >= 4) LAUNCH(float, 2);
        else LAUNCH(float, 1);
    } else {
        if (a->S >= 16) LAUNCH(Bf16, 8);
        else if (a->S >= 4) LAUNCH(Bf16, 2);
        else LAUNCH(Bf16, 1);
    }
#undef LAUNCH
    hipLaunchKernelGGL(k_scalars, dim3(1), dim3(kScalarThreads), 0, s, &sc->partials[0][0], grid, &sc->book, a->lr_table, sa);
    if (vec == 4) hipLaunchKernelGGL(k_flat_finish<4>, dim3(grid), dim3(kThreads), 0, s, sc, (long long)a->numel, n_tiles, user);
    else hipLaunchKernelGGL(k_flat_finish<8>, dim3(grid), dim3(kThreads), 0, s, sc, (long long)a->numel, n_tiles, user);
    HIP_TRY(nullptr, hipGetLastError());
    return ADASCALE_OK;
}

int adascale_profile_begin(adascale_ctx *c, int32_t max_steps)
{
    if (!c) return ADASCALE_EINVAL;
    if (max_steps < 1 || max_steps > 100000) return fail(c, ADASCALE_EINVAL, "max_steps out of range");
    DeviceGuard guard;
    HIP_TRY(c, guard.enter(c->cfg.device));
    while ((int)c->prof_ev.size() < 4 * max_steps) {
        hipEvent_t e;
        HIP_TRY(c, hipEventCreate(&e));
        c->prof_ev.push_back(e);
    }
    c->prof_cap = max_steps;
    c->prof_n = 0;
    c->prof_on = true;
    return ADASCALE_OK;
}

int adascale_profile_end(adascale_ctx *c, double ms[3], int32_t *n_steps)
{
    if (!c) return ADASCALE_EINVAL;
    if (!ms || !n_steps) return fail(c, ADASCALE_EINVAL, "null output");
    if (!c->prof_on) return fail(c, ADASCALE_ESTATE, "profiling is not on");
    c->prof_on = false;
    ms[0] = ms[1] = ms[2] = 0.0;
    *n_steps = c->prof_n;
    if (c->prof_n == 0) return ADASCALE_OK;
    DeviceGuard guard;
    HIP_TRY(c, guard.enter(c->cfg.device));
    HIP_TRY(c, hipEventSynchronize(c->prof_ev[(size_t)4 * (c->prof_n - 1) + 3]));
    for (int i = 0; i < c->prof_n; ++i)
        for (int j = 0; j < 3; ++j) {
            float t = 0.f;
            HIP_TRY(c, hipEventElapsedTime(&t, c->prof_ev[(size_t)4 * i + j], c->prof_ev[(size_t)4 * i + j + 1]));
            ms[j] += t;
        }
    for (int j = 0; j < 3; ++j) ms[j] /= c->prof_n;
    return ADASCALE_OK;
}

}  // extern "C"
