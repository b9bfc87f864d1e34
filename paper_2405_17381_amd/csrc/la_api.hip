// C ABI of the library: argument checks, launch planning and kernel launches.
// Declarations and the contract of every entry point are in include/la.h.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <mutex>

#include "la_common.h"
#include "la_debug.h"
#include "la_kernels_bf16.h"
#include "la_kernels_bf16_dma.h"
#include "la_kernels_bf16_dma_wide.h"
#include "la_kernels_f32.h"
#include "la_kernels_f32m.h"
#include "la_kernels_gate.h"
#include "la_kernels_lrpe.h"
#include "la_kernels_misc.h"
#include "la_kernels_prepass.h"

// Scratch of la_fwd_static: the segment states of one forward call.  One copy per GPU the
// library runs on, held until the process ends.  In host code this name is only a handle
// for hipGetSymbolAddress; the device address it yields is what the kernels are given.
static __device__ __align__(256) unsigned char la_static_scratch[LA_STATIC_SCRATCH_BYTES];

namespace {

// Device address of la_static_scratch on each GPU, looked up once per device.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};

int static_scratch(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return LA_ERR_LAUNCH;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(la_static_scratch)) != hipSuccess || !ptr) return LA_ERR_LAUNCH;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return LA_OK;
}

// Test / tuning switches.  They are process-wide, start at zero, never look at the
// environment and change only through la_debug_set (la_debug.h, not part of the public
// header): the workspace query and the launch that follows therefore always plan alike.
struct Switches {
    std::atomic<long> lseg{0};           // > 0: segment length in tokens
    std::atomic<long> no_pair{0};        // != 0: the dK and dV scans are launched separately
    std::atomic<long> no_decay_skip{0};  // != 0: the segment-state pre-pass reads every block
    std::atomic<long> f32_plain{0};      // != 0: fp32 at d = 128 runs the FMA kernel
    std::atomic<long> store_policy{0};   // direct-to-LDS scan: 2 = ordinary instead of non-temporal result stores
    std::atomic<long> staged_prepass{0}; // != 0: bf16 runs the register-staged segment-state pre-pass
    std::atomic<long> prepass_groups{0}; // 1, 2: wave groups per workgroup of the direct-to-LDS pre-pass (own choice: 4)
    std::atomic<long> no_trio{0};        // != 0: la_bwd's direct-to-LDS block scans as a dQ launch and a paired dK / dV launch
    std::atomic<long> wide_slices{0};    // != 0: la_fwd_wide always runs accumulated scans over d_v-wide slices
    std::atomic<long> ablate{0};         // 1..4: measurement-only variants of the direct-to-LDS scan
    std::atomic<long> staged_scan{0};    // != 0: bf16 runs the register-staged block scan
                                         // (64-row blocks) instead of the direct-to-LDS one (32-row)
} g_sw;

std::atomic<long> *find_switch(const char *name)
{
    if (!name) return nullptr;
    if (!std::strcmp(name, "lseg")) return &g_sw.lseg;
    if (!std::strcmp(name, "no_pair")) return &g_sw.no_pair;
    if (!std::strcmp(name, "no_decay_skip")) return &g_sw.no_decay_skip;
    if (!std::strcmp(name, "f32_plain")) return &g_sw.f32_plain;
    if (!std::strcmp(name, "staged_scan")) return &g_sw.staged_scan;
    if (!std::strcmp(name, "ablate")) return &g_sw.ablate;
    if (!std::strcmp(name, "wide_slices")) return &g_sw.wide_slices;
    if (!std::strcmp(name, "no_trio")) return &g_sw.no_trio;
    if (!std::strcmp(name, "staged_prepass")) return &g_sw.staged_prepass;
    if (!std::strcmp(name, "prepass_groups")) return &g_sw.prepass_groups;
    if (!std::strcmp(name, "store_policy")) return &g_sw.store_policy;
    return nullptr;
}

// MI355X: 256 compute units.  The planner is pure host arithmetic on purpose
// (the workspace query must give the same answer with or without a GPU).
constexpr int kComputeUnits = 256;
// A sequence is cut into segments only when there are fewer (batch, head) scans
// than compute units; it is then cut finely enough for two workgroups per unit.
// Measured on the 64K-token sweep: one workgroup per unit without the segment-
// state pre-pass beats two per unit with it, and 2048-token segments are best
// among 512..8192.
// bf16 at d = 64 runs two-wave workgroups, four to a unit: measured at 64 and 32 scans of 32K and
// 64K tokens, 2048-token segments (1024 workgroups) beat 4096-token ones (512) by 3 to 5 %.
constexpr int kTargetWorkgroups = 2 * kComputeUnits;
constexpr int kTargetWorkgroupsBf16D64 = 4 * kComputeUnits;
constexpr int kMinSegmentTokens = 512;

struct Plan {
    int tile;       // block length BK (the paper's "block size B")
    int L;          // segment length in tokens (multiple of tile)
    int S;          // segments per scan
};

// Block length of the block-scan kernel la_fwd / la_bwd run (the paper's "block size B").
int tile_len(int d, la_dtype dt)
{
    if (dt == LA_BF16) return g_sw.staged_scan.load(std::memory_order_relaxed) ? 64 : 32;
    return d == 64 ? 64 : 32;
}

// Segment lengths are multiples of this: the longest block any kernel of the path uses
// (the bf16 segment-state pre-pass and the extended scan variants work on 64-row blocks).
int segment_granule(int d, la_dtype dt) { return dt == LA_BF16 ? 64 : tile_len(d, dt); }

int round_up(int x, int m) { return (x + m - 1) / m * m; }

Plan make_plan(int B, int H, int n, int d, la_dtype dt)
{
    Plan p;
    p.tile = tile_len(d, dt);
    const int gran = segment_granule(d, dt);
    const long scans = (long)B * H;
    int L = round_up(n, gran);
    if (scans < kComputeUnits) {
        const bool small_wgs = dt == LA_BF16 && d == 64 && !g_sw.staged_scan.load(std::memory_order_relaxed);
        const long target = small_wgs ? kTargetWorkgroupsBf16D64 : kTargetWorkgroups;
        const long want = (target + scans - 1) / scans;              // segments wanted per scan
        long l = (n + want - 1) / want;
        if (l < kMinSegmentTokens) l = kMinSegmentTokens;
        l = round_up((int)l, gran);
        if (l < L) L = (int)l;
    }
    // tuning / test override: segment length in tokens
    long v = g_sw.lseg.load(std::memory_order_relaxed);
    if (v > 0 && scans <= 65535) {              // the segment scan's grid has one row per scan
        v = round_up((int)(v > (1 << 30) ? (1 << 30) : v), gran);
        L = (int)(v < round_up(n, gran) ? v : round_up(n, gran));
    }
    p.L = L;
    p.S = (int)(((long)n + L - 1) / L);
    return p;
}

int check_common(int B, int H, int n, int d, la_dtype dt)
{
    if (dt != LA_F32 && dt != LA_BF16) return LA_ERR_DTYPE;
    if (B < 1 || H < 1 || n < 1 || H > LA_MAX_HEADS) return LA_ERR_SHAPE;
    if (n > LA_MAX_SEQ_LEN) return LA_ERR_SHAPE;        // keeps round_up(n, tile) and seg_lo + L (< 2 n) in int
    if (d != 64 && d != 128) return LA_ERR_SHAPE;
    if ((long)B * H > (long)INT32_MAX / 4096) return LA_ERR_SHAPE;
    return LA_OK;
}

int check_lambda(const float *lambda, int H, LaLambdas *out)
{
    for (int h = 0; h < H; ++h) {
        const float l = lambda[h];
        if (!std::isfinite(l) || !(l > 0.0f) || !(l <= 1.0f)) return LA_ERR_LAMBDA;
        out->v[h] = l;
        out->lg2[h] = (float)std::log2((double)l);
    }
    for (int h = H; h < LA_MAX_HEADS; ++h) { out->v[h] = 1.0f; out->lg2[h] = 0.0f; }
    // heads by decreasing lambda (stable): insertion sort, H <= 256
    for (int h = 0; h < LA_MAX_HEADS; ++h) out->order[h] = (uint8_t)h;
    for (int i = 1; i < H; ++i) {
        const uint8_t x = out->order[i];
        int j = i - 1;
        while (j >= 0 && out->v[out->order[j]] < out->v[x]) { out->order[j + 1] = out->order[j]; --j; }
        out->order[j + 1] = x;
    }
    return LA_OK;
}

bool aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }

size_t state_bytes(const Plan &p, int B, int H, int d)
{
    if (p.S <= 1) return 0;
    return (size_t)B * H * p.S * (size_t)d * d * sizeof(float);
}

// ---- profiling hooks (single benchmarking thread) ---------------------------
// The events are created by la_profile_enable, never inside a forward / backward call:
// a call only records into events that already exist.
struct Profile {
    bool on = false;
    int count = 0;
    hipEvent_t start[LA_PROFILE_MAX_LAUNCHES];
    hipEvent_t stop[LA_PROFILE_MAX_LAUNCHES];
    int created = 0;
} g_prof;

struct ScopedTimer {
    hipStream_t s;
    int slot = -1;
    explicit ScopedTimer(hipStream_t st) : s(st)
    {
        if (!g_prof.on || g_prof.count >= g_prof.created) return;
        slot = g_prof.count++;
        (void)hipEventRecord(g_prof.start[slot], s);
    }
    ~ScopedTimer() { if (slot >= 0) (void)hipEventRecord(g_prof.stop[slot], s); }
};

// ---- kernel launch helpers ----------------------------------------------------
template <typename K>
hipError_t allow_lds(K kernel, size_t bytes)
{
    return hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

template <int D, bool REV, bool ACT>
hipError_t launch_bf16(const ScanLaunch &a, const LaLambdas &lams, hipStream_t s)
{
    using Cfg = Bf16Cfg<D>;
    auto kern = la_scan_bf16<D, REV, ACT>;
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(once, [&] { attr_err = allow_lds(kern, Cfg::lds_bytes); });
    if (attr_err != hipSuccess) return attr_err;
    // paired launch: two workgroups per item, items padded to a multiple of the 8 XCDs
    const unsigned wgs = a.nroles == 2 ? 2u * (unsigned)((a.items + 7) / 8 * 8) : (unsigned)a.items;
    dim3 grid(wgs), block(Cfg::NT);
    hipLaunchKernelGGL(kern, grid, block, Cfg::lds_bytes, s, a, lams);
    return hipGetLastError();
}

// The backward pass's three block scans in one launch (see the kernel).
template <bool STRIDED, int D = 128>
hipError_t launch_bf16_dma_trio(const ScanLaunch &a, const LaLambdas &lams, hipStream_t s)
{
    using Cfg = DmaCfg<3, D>;
    auto kern = la_scan_bf16_dma<false, true, 0, 3, true, STRIDED, D>;
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(once, [&] { attr_err = allow_lds(kern, Cfg::lds_bytes); });
    if (attr_err != hipSuccess) return attr_err;
    dim3 grid(3u * (unsigned)((a.items + 7) / 8 * 8)), block(Cfg::NT);
    hipLaunchKernelGGL(kern, grid, block, Cfg::lds_bytes, s, a, lams);
    return hipGetLastError();
}

template <bool REV, bool NT_STORE, int ABL, int NS = 3, bool STRIDED = false, int D = 128>
hipError_t launch_bf16_dma_variant(const ScanLaunch &a, const LaLambdas &lams, hipStream_t s)
{
    using Cfg = DmaCfg<NS, D>;
    auto kern = la_scan_bf16_dma<REV, NT_STORE, ABL, NS, false, STRIDED, D>;
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(once, [&] { attr_err = allow_lds(kern, Cfg::lds_bytes); });
    if (attr_err != hipSuccess) return attr_err;
    // paired launch: two workgroups per item, items padded to a multiple of the 8 XCDs
    const unsigned wgs = a.nroles == 2 ? 2u * (unsigned)((a.items + 7) / 8 * 8) : (unsigned)a.items;
    dim3 grid(wgs), block(Cfg::NT);
    hipLaunchKernelGGL(kern, grid, block, Cfg::lds_bytes, s, a, lams);
    return hipGetLastError();
}

// Cache policy of the result stores: non-temporal.  Timed alone, a single-scan launch is 8 %
// faster with ordinary stores, but only because L2 then hands part of its write-back to
// whatever runs next: over a forward + backward sequence non-temporal stores in all three
// launches win by 6 % ("store_policy" switch = 2 selects ordinary stores, for measurements).
template <bool REV, bool STRIDED = false, int D = 128>
hipError_t launch_bf16_dma(const ScanLaunch &a, const LaLambdas &lams, hipStream_t s)
{
    const bool nt = g_sw.store_policy.load(std::memory_order_relaxed) != 2;
    // operands with their own layouts (strided entry points, slices of wider rows), and d = 64: one variant
    if (STRIDED || D != 128) return launch_bf16_dma_variant<REV, true, 0, 3, STRIDED, D>(a, lams, s);
    switch (g_sw.ablate.load(std::memory_order_relaxed)) {
    case 1: return launch_bf16_dma_variant<REV, true, 1>(a, lams, s);
    case 2: return launch_bf16_dma_variant<REV, true, 2>(a, lams, s);
    case 3: return launch_bf16_dma_variant<REV, true, 3>(a, lams, s);
    case 4: return nt ? launch_bf16_dma_variant<REV, true, 4>(a, lams, s)
                      : launch_bf16_dma_variant<REV, false, 4>(a, lams, s);
    default: break;
    }
    return nt ? launch_bf16_dma_variant<REV, true, 0>(a, lams, s)
              : launch_bf16_dma_variant<REV, false, 0>(a, lams, s);
}

template <int G, bool STRIDED = false, int D = 128>
hipError_t launch_prepass_bf16_dma(const ScanLaunch &a, const LaLambdas &lams, hipStream_t s)
{
    using Cfg = DmaPrepassCfg<G, D>;
    auto kern = la_prepass_bf16_dma<G, STRIDED, D>;
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(once, [&] { attr_err = allow_lds(kern, Cfg::lds_bytes); });
    if (attr_err != hipSuccess) return attr_err;
    dim3 grid((unsigned)(a.items * a.nroles)), block(Cfg::NT);
    hipLaunchKernelGGL(kern, grid, block, Cfg::lds_bytes, s, a, lams);
    return hipGetLastError();
}

template <int D, bool ACT>
hipError_t launch_prepass_bf16(const ScanLaunch &a, const LaLambdas &lams, hipStream_t s)
{
    using Cfg = PrepassCfg<D>;
    auto kern = la_prepass_bf16<D, ACT>;
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(once, [&] { attr_err = allow_lds(kern, Cfg::lds_bytes); });
    if (attr_err != hipSuccess) return attr_err;
    dim3 grid((unsigned)(a.items * a.nroles)), block(Cfg::NT);
    hipLaunchKernelGGL(kern, grid, block, Cfg::lds_bytes, s, a, lams);
    return hipGetLastError();
}

template <int D, int BK, bool REV, bool STATE_ONLY>
hipError_t launch_f32(const ScanLaunch &a, const LaLambdas &lams, hipStream_t s)
{
    using Cfg = F32Cfg<D, BK>;
    auto kern = la_scan_f32<D, BK, REV, STATE_ONLY>;
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(once, [&] { attr_err = allow_lds(kern, Cfg::lds_bytes); });
    if (attr_err != hipSuccess) return attr_err;
    dim3 grid((unsigned)(a.items * a.nroles)), block(Cfg::NT);   // roles one after the other
    hipLaunchKernelGGL(kern, grid, block, Cfg::lds_bytes, s, a, lams);
    return hipGetLastError();
}

template <int D, bool REV, bool STATE_ONLY>
hipError_t launch_f32m(const ScanLaunch &a, const LaLambdas &lams, hipStream_t s)
{
    using Cfg = F32mCfg<D>;
    auto kern = la_scan_f32m<D, REV, STATE_ONLY>;
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(once, [&] { attr_err = allow_lds(kern, Cfg::lds_bytes); });
    if (attr_err != hipSuccess) return attr_err;
    dim3 grid((unsigned)(a.items * a.nroles)), block(Cfg::NT);   // roles one after the other
    hipLaunchKernelGGL(kern, grid, block, Cfg::lds_bytes, s, a, lams);
    return hipGetLastError();
}

// bf16, direct-to-LDS family: plain launches and launches whose operands have their own layouts
template <bool REV, bool STATE_ONLY, int D>
hipError_t launch_bf16_direct(const ScanLaunch &a, const LaLambdas &lams, bool strided, hipStream_t s)
{
    if (STATE_ONLY) {
        if (strided) return launch_prepass_bf16_dma<4, true, D>(a, lams, s);
        if constexpr (D == 128) {
            switch (g_sw.prepass_groups.load(std::memory_order_relaxed)) {
            case 1: return launch_prepass_bf16_dma<1, false, D>(a, lams, s);
            case 2: return launch_prepass_bf16_dma<2, false, D>(a, lams, s);
            default: break;
            }
        }
        return launch_prepass_bf16_dma<4, false, D>(a, lams, s);
    }
    return strided ? launch_bf16_dma<REV, true, D>(a, lams, s) : launch_bf16_dma<REV, false, D>(a, lams, s);
}

// bf16, register-staged family (64-row blocks): every activation / accumulation variant, and
// everything when the "staged_scan" switch is set
template <bool REV, bool STATE_ONLY, int D>
hipError_t launch_bf16_staged(const ScanLaunch &a, const LaLambdas &lams, bool ext, hipStream_t s)
{
    if (STATE_ONLY) return ext ? launch_prepass_bf16<D, true>(a, lams, s) : launch_prepass_bf16<D, false>(a, lams, s);
    return ext ? launch_bf16<D, REV, true>(a, lams, s) : launch_bf16<D, REV, false>(a, lams, s);
}

template <bool REV, bool STATE_ONLY>
hipError_t launch_scan_kernel(const ScanLaunch &a, const LaLambdas &lams, int d,
                              la_dtype dt, hipStream_t s)
{
    if (dt == LA_BF16) {
        // LA_ACT_EXT alone: operands with their own layouts, nothing else; any other bit: an
        // activation or an accumulating epilogue, which only the register-staged kernels carry
        const int acts = a.r[0].act | a.r[a.nroles - 1].act;
        const bool plain = acts == 0 || acts == LA_ACT_EXT;
        const bool staged = !plain || g_sw.staged_scan.load(std::memory_order_relaxed) != 0 ||
                            (STATE_ONLY && g_sw.staged_prepass.load(std::memory_order_relaxed) != 0);
        if (staged)
            return d == 64 ? launch_bf16_staged<REV, STATE_ONLY, 64>(a, lams, acts != 0, s)
                           : launch_bf16_staged<REV, STATE_ONLY, 128>(a, lams, acts != 0, s);
        return d == 64 ? launch_bf16_direct<REV, STATE_ONLY, 64>(a, lams, acts != 0, s)
                       : launch_bf16_direct<REV, STATE_ONLY, 128>(a, lams, acts != 0, s);
    }
    // fp32: d = 64 runs the literal FMA kernel with 64-row blocks; d = 128 the matrix-core kernel
    // (32-row blocks; the "f32_plain" switch selects the FMA kernel there too, for comparisons)
    if (d == 64) return launch_f32<64, 64, REV, STATE_ONLY>(a, lams, s);
    if (g_sw.f32_plain.load(std::memory_order_relaxed)) return launch_f32<128, 32, REV, STATE_ONLY>(a, lams, s);
    return launch_f32m<128, REV, STATE_ONLY>(a, lams, s);
}

LaLayout contiguous_layout(int H, int n, int d)
{
    LaLayout l;
    l.bs = (long)H * n * d; l.hs = (long)n * d; l.ld = d;
    return l;
}

// How the query / key operands of a call differ from plain contiguous [B, H, n, d] tensors.
struct Variant {
    bool swish = false;     // Q, K are pre-activations (la_fwd_swish / la_bwd_swish)
    int wide_ld = 0;        // > 0: Q, K (and dQ, dK) are d-wide slices of rows this many elements wide
    bool accumulate = false; // the result over this slice is added to O (forward) / dV (backward)
    // caller-given layouts (la_*_strided): Q, K, V / O (forward); Q, K, V / dO / dQ, dK, dV (backward)
    const LaLayout *in = nullptr, *out = nullptr, *dout = nullptr;
    // backward only: the segment states la_fwd left in its workspace for the same problem
    // (la_bwd_saved); the dQ scan reads them transposed instead of recomputing them
    const float *fwd_states = nullptr;
};

ScanArgs make_args(const void *A, const void *Bm, const void *C, void *Out, const Plan &p,
                   int H, int n, int d, la_dtype dt, float *states, int transpose_init)
{
    ScanArgs a;
    a.lA = a.lB = a.lC = a.lO = a.lE = contiguous_layout(H, n, d);
    a.A = A; a.Bm = Bm; a.C = C; a.Out = Out;
    a.states = p.S > 1 ? states : nullptr;
    a.n = n; a.H = H; a.L = p.L; a.S = p.S;
    a.B = 0;             // set by the callers that launch a pre-pass
    a.transpose_init = transpose_init;
    // Decay cut-off: contributions weighted below 2^-bits of the nearest row's weight are
    // not read.  fp32: 2^-48, far below the 2^-24 resolution of the state they would be
    // added to; bf16: 2^-32, far below both that and the 2^-8 resolution of the bf16
    // operand the state is rounded to when it is used (the "no_decay_skip" switch reads everything).
    a.skip_bits = g_sw.no_decay_skip.load(std::memory_order_relaxed) ? 0.0f : (dt == LA_BF16 ? 32.0f : 48.0f);
    a.rev = 0;
    a.st_in = nullptr;
    a.st_out = nullptr;
    a.act = 0;
    a.E = nullptr;
    return a;
}

// Segment-state pre-pass: the local end state of every segment of scan(., Bm, C),
// for one scan or, in one launch, for two independent scans (their short, latency-
// bound chains then fill the machine together).
int run_prepass(const ScanArgs *a, int nroles, const LaLambdas &lams, long scans, int d, la_dtype dt,
                hipStream_t s)
{
    ScanLaunch l = {};
    l.r[0] = a[0]; l.r[1] = a[nroles - 1]; l.nroles = nroles; l.items = (int)(scans * a[0].S);
    return launch_scan_kernel<false, true>(l, lams, d, dt, s) == hipSuccess ? LA_OK : LA_ERR_LAUNCH;
}

// Exclusive scan over the segments, in place: local states -> entering states.
SegScanArgs segment_scan_args(const ScanArgs &a, bool rev, int d)
{
    SegScanArgs sa;
    sa.states = a.states; sa.init = rev ? nullptr : a.st_in; sa.skip_bits = a.skip_bits;
    sa.H = a.H; sa.S = a.S; sa.L = a.L; sa.DD = d * d;
    return sa;
}

template <bool REV>
int run_segment_scan(const ScanArgs &a, const LaLambdas &lams, long scans, int d, hipStream_t s)
{
    dim3 grid((unsigned)((d * d / 4 + 255) / 256), (unsigned)scans), block(256);
    hipLaunchKernelGGL(la_segment_scan<REV>, grid, block, 0, s, segment_scan_args(a, REV, d), lams);
    return hipGetLastError() == hipSuccess ? LA_OK : LA_ERR_LAUNCH;
}

// The backward pass's forward and reverse segment scans as one launch.
int run_segment_scan_pair(const ScanArgs &f, const ScanArgs &r, const LaLambdas &lams, long scans, int d,
                          hipStream_t s)
{
    dim3 grid((unsigned)((d * d / 4 + 255) / 256), (unsigned)scans, 2), block(256);
    hipLaunchKernelGGL(la_segment_scan_pair, grid, block, 0, s, segment_scan_args(f, false, d),
                       segment_scan_args(r, true, d), lams);
    return hipGetLastError() == hipSuccess ? LA_OK : LA_ERR_LAUNCH;
}

template <bool REV>
int run_block_scan(const ScanArgs &a, const LaLambdas &lams, long scans, int d, la_dtype dt, hipStream_t s)
{
    ScanLaunch l = {};
    l.r[0] = a; l.r[1] = a; l.nroles = 1; l.items = (int)(scans * a.S);
    ScopedTimer t(s);
    return launch_scan_kernel<REV, false>(l, lams, d, dt, s) == hipSuccess ? LA_OK : LA_ERR_LAUNCH;
}

// One decayed causal scan Out = scan(A, Bm, C): [pre-pass -> segment scan ->] block scan.
template <bool REV>
int run_scan(const void *A, const void *Bm, const void *C, void *Out, const LaLambdas &lams,
             const Plan &p, int B, int H, int n, int d, la_dtype dt, float *states, hipStream_t s,
             const float *st_in = nullptr, float *st_out = nullptr, const Variant &var = Variant())
{
    const long scans = (long)B * H;
    ScanArgs a = make_args(A, Bm, C, Out, p, H, n, d, dt, states, 0);
    // forward use only (O = scan(Q, K, V)): A and Bm are the query / key operands
    if (var.swish) a.act |= LA_ACT_A | LA_ACT_BM;
    if (var.wide_ld > 0) {
        a.lA = a.lB = contiguous_layout(H, n, var.wide_ld);
        a.act |= LA_ACT_EXT | (var.accumulate ? LA_ACT_ACC : 0);
    }
    if (var.in) {
        a.lA = a.lB = a.lC = *var.in;
        a.lO = *var.out;
        a.act |= LA_ACT_EXT;
    }
    a.B = B;
    a.rev = REV ? 1 : 0;
    a.st_in = st_in;
    a.st_out = st_out;
    if (p.S > 1) {
        int rc = run_prepass(&a, 1, lams, scans, d, dt, s);
        if (rc == LA_OK) rc = run_segment_scan<REV>(a, lams, scans, d, s);
        if (rc != LA_OK) return rc;
    }
    return run_block_scan<REV>(a, lams, scans, d, dt, s);
}

// The two reverse scans of Alg. 6's second loop,
//     dK = scan_rev(V, dO, Q)   (state  sum w dO^T Q = dKV^T)
//     dV = scan_rev(K, Q, dO)   (state  sum w Q^T dO = dKV),
// share one set of segment states (dV reads dK's transposed) and, on the bf16
// path, one paired launch in which the two workgroups of a segment sit on the
// same XCD, so that dO and Q, which both read, come from HBM once.
int run_reverse_pair(const ScanArgs &ak, const ScanArgs &av, const LaLambdas &lams, long scans,
                     int d, la_dtype dt, hipStream_t s)
{
    ScanLaunch l = {};
    l.items = (int)(scans * ak.S);
    const bool pair = dt == LA_BF16 && g_sw.no_pair.load(std::memory_order_relaxed) == 0;
    if (pair) {
        l.r[0] = ak; l.r[1] = av; l.nroles = 2;
        ScopedTimer t(s);
        return launch_scan_kernel<true, false>(l, lams, d, dt, s) == hipSuccess ? LA_OK : LA_ERR_LAUNCH;
    }
    int rc = run_block_scan<true>(ak, lams, scans, d, dt, s);
    if (rc != LA_OK) return rc;
    return run_block_scan<true>(av, lams, scans, d, dt, s);
}

// Backward pass.  dQ = scan(dO, V, K) is the first loop of Alg. 6 (state KV^T); the
// second loop is the reverse pair above.  With segments, the two pre-passes (forward
// states of (V, K), reverse states of (dO, Q)) run as one launch into the two halves
// of the scratch, then the two segment scans, then the block scans: for bf16 at d = 128
// without activations all three as the roles of one launch, else dQ's and the pair's.
// With `swish`, Q and K are pre-activations: they are activated wherever they are an
// operand, and dQ, dK are multiplied by phi'(Q), phi'(K) as they are stored.
int run_backward(const void *Q, const void *K, const void *V, const void *dO, void *dQ, void *dK,
                 void *dV, const LaLambdas &lams, const Plan &p, int B, int H, int n, int d,
                 la_dtype dt, float *ws, hipStream_t s, const Variant &var)
{
    const long scans = (long)B * H;
    // la_fwd's states are those of scan(., K, V); the dQ scan wants scan(., V, K): the transposes
    const bool reuse = var.fwd_states != nullptr && p.S > 1;
    float *ws_f = reuse ? const_cast<float *>(var.fwd_states) : ws;
    float *ws_r = reuse ? ws : (ws ? ws + (size_t)scans * p.S * (size_t)d * d : nullptr);
    ScanArgs pre[2];
    pre[0] = make_args(dO, V, K, dQ, p, H, n, d, dt, ws_f, reuse ? 1 : 0);
    pre[1] = make_args(V, dO, Q, dK, p, H, n, d, dt, ws_r, 0);
    pre[1].rev = 1;
    pre[0].B = pre[1].B = B;
    ScanArgs av = make_args(K, Q, dO, dV, p, H, n, d, dt, ws_r, 1);
    av.rev = 1;
    if (var.swish) {
        pre[0].act = LA_ACT_C | LA_ACT_OUT; pre[0].E = Q;      // dQ = scan(dO, V, phi(K)) * phi'(Q)
        pre[1].act = LA_ACT_C | LA_ACT_OUT; pre[1].E = K;      // dK = scan_rev(V, dO, phi(Q)) * phi'(K)
        av.act = LA_ACT_A | LA_ACT_BM;                         // dV = scan_rev(phi(K), phi(Q), dO)
    }
    if (var.wide_ld > 0) {
        // Q, K, dQ, dK are d-wide slices of wider rows; dV sums over the slices
        const LaLayout w = contiguous_layout(H, n, var.wide_ld);
        pre[0].lC = pre[0].lO = w;                             // dQ slice = scan(dO, V, K slice)
        pre[1].lC = pre[1].lO = w;                             // dK slice = scan_rev(V, dO, Q slice)
        av.lA = av.lB = w;                                     // dV (+)= scan_rev(K slice, Q slice, dO)
        pre[0].act |= LA_ACT_EXT; pre[1].act |= LA_ACT_EXT;
        av.act |= LA_ACT_EXT | (var.accumulate ? LA_ACT_ACC : 0);
    }
    if (var.in) {
        pre[0].lA = *var.dout; pre[0].lB = pre[0].lC = *var.in; pre[0].lO = *var.out;   // scan(dO, V, K) -> dQ
        pre[1].lA = *var.in; pre[1].lB = *var.dout; pre[1].lC = *var.in; pre[1].lO = *var.out;  // (V, dO, Q) -> dK
        av.lA = av.lB = *var.in; av.lC = *var.dout; av.lO = *var.out;                   // (K, Q, dO) -> dV
        pre[0].act |= LA_ACT_EXT; pre[1].act |= LA_ACT_EXT; av.act |= LA_ACT_EXT;
    }
    if (p.S > 1) {
        int rc;
        if (reuse) {
            rc = run_prepass(&pre[1], 1, lams, scans, d, dt, s);
            if (rc == LA_OK) rc = run_segment_scan<true>(pre[1], lams, scans, d, s);
        } else {
            rc = run_prepass(pre, 2, lams, scans, d, dt, s);
            if (rc == LA_OK) rc = run_segment_scan_pair(pre[0], pre[1], lams, scans, d, s);
        }
        if (rc != LA_OK) return rc;
    }
    const int acts = pre[0].act | pre[1].act | av.act;
    const bool all_ext = pre[0].act == LA_ACT_EXT && pre[1].act == LA_ACT_EXT && av.act == LA_ACT_EXT;
    if (!g_sw.no_trio.load(std::memory_order_relaxed) && dt == LA_BF16 &&
        (acts == 0 || all_ext) && !g_sw.staged_scan.load(std::memory_order_relaxed) &&
        !g_sw.no_pair.load(std::memory_order_relaxed) && !g_sw.ablate.load(std::memory_order_relaxed)) {
        ScanLaunch l;
        l.r[0] = pre[0]; l.r[1] = pre[1]; l.r[2] = av; l.nroles = 3; l.items = (int)(scans * p.S);
        ScopedTimer t(s);
        hipError_t e;
        if (d == 64) e = all_ext ? launch_bf16_dma_trio<true, 64>(l, lams, s) : launch_bf16_dma_trio<false, 64>(l, lams, s);
        else e = all_ext ? launch_bf16_dma_trio<true>(l, lams, s) : launch_bf16_dma_trio<false>(l, lams, s);
        return e == hipSuccess ? LA_OK : LA_ERR_LAUNCH;
    }
    // Two launches.  The reversed pair goes first: it ends at the segments' first rows, where the
    // dQ scan starts, so what the Infinity Cache still holds of K, V, dO is what dQ reads first
    // (measured with cold caches, bf16 d = 128: la_bwd 0.54 against 0.56 ms in the other order).
    int rc = run_reverse_pair(pre[1], av, lams, scans, d, dt, s);
    if (rc != LA_OK) return rc;
    return run_block_scan<false>(pre[0], lams, scans, d, dt, s);
}

int check_workspace(const Plan &p, int B, int H, int d, void *workspace, size_t workspace_bytes,
                    bool is_bwd)
{
    // one workgroup per (scan, segment) and role, up to three roles in a launch: keep the grid within 2^31
    if ((long)B * H * p.S > (1L << 29)) return LA_ERR_SHAPE;
    const size_t need = state_bytes(p, B, H, d) * (is_bwd ? 2 : 1);
    if (need == 0) return LA_OK;
    if (workspace == nullptr || ((uintptr_t)workspace & 255u) != 0 || workspace_bytes < need)
        return LA_ERR_WORKSPACE;
    return LA_OK;
}

template <bool BWD>
int run_gate_norm(const GateArgs &g, int B, int n, int d, la_dtype dt, hipStream_t s)
{
    dim3 grid((unsigned)((n + 7) / 8), (unsigned)B), block(256);
    if (dt == LA_BF16) {
        if (d == 64) hipLaunchKernelGGL((la_gate_norm_kernel<64, true, BWD>), grid, block, 0, s, g);
        else hipLaunchKernelGGL((la_gate_norm_kernel<128, true, BWD>), grid, block, 0, s, g);
    } else {
        if (d == 64) hipLaunchKernelGGL((la_gate_norm_kernel<64, false, BWD>), grid, block, 0, s, g);
        else hipLaunchKernelGGL((la_gate_norm_kernel<128, false, BWD>), grid, block, 0, s, g);
    }
    return hipGetLastError() == hipSuccess ? LA_OK : LA_ERR_LAUNCH;
}

template <bool BWD>
int run_lrpe(const LrpeArgs &a, int B, int d, la_dtype dt, hipStream_t s)
{
    dim3 grid((unsigned)a.tiles, (unsigned)(B * a.H)), block(256);
    if (dt == LA_BF16) {
        if (d == 64) hipLaunchKernelGGL((la_lrpe_rotate_kernel<64, true, BWD>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((la_lrpe_rotate_kernel<128, true, BWD>), grid, block, 0, s, a);
    } else {
        if (d == 64) hipLaunchKernelGGL((la_lrpe_rotate_kernel<64, false, BWD>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((la_lrpe_rotate_kernel<128, false, BWD>), grid, block, 0, s, a);
    }
    return hipGetLastError() == hipSuccess ? LA_OK : LA_ERR_LAUNCH;
}

// Argument checks and planning shared by the forward entry points.
int forward(const void *Q, const void *K, const void *V, const float *lambda, void *O,
            const float *kv_in, float *kv_out, int B, int H, int n, int d, la_dtype dt,
            void *workspace, size_t workspace_bytes, void *hip_stream, const Variant &var)
{
    int rc = check_common(B, H, n, d, dt);
    if (rc != LA_OK) return rc;
    if (!Q || !K || !V || !O || !lambda) return LA_ERR_NULL;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O) ||
        !aligned16(kv_in) || !aligned16(kv_out)) return LA_ERR_ALIGN;
    LaLambdas lams;
    rc = check_lambda(lambda, H, &lams);
    if (rc != LA_OK) return rc;
    const Plan p = make_plan(B, H, n, d, dt);
    rc = check_workspace(p, B, H, d, workspace, workspace_bytes, false);
    if (rc != LA_OK) return rc;
    hipStream_t s = (hipStream_t)hip_stream;
    // O = scan(Q, K, V)                                                   (Alg. 5)
    return run_scan<false>(Q, K, V, O, lams, p, B, H, n, d, dt, (float *)workspace, s, kv_in, kv_out, var);
}

// ... and by the backward entry points.
int backward(const void *Q, const void *K, const void *V, const float *lambda, const void *dO,
             void *dQ, void *dK, void *dV, int B, int H, int n, int d, la_dtype dt,
             void *workspace, size_t workspace_bytes, void *hip_stream, const Variant &var)
{
    int rc = check_common(B, H, n, d, dt);
    if (rc != LA_OK) return rc;
    if (!Q || !K || !V || !dO || !dQ || !dK || !dV || !lambda) return LA_ERR_NULL;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(dO) ||
        !aligned16(dQ) || !aligned16(dK) || !aligned16(dV)) return LA_ERR_ALIGN;
    LaLambdas lams;
    rc = check_lambda(lambda, H, &lams);
    if (rc != LA_OK) return rc;
    const Plan p = make_plan(B, H, n, d, dt);
    rc = check_workspace(p, B, H, d, workspace, workspace_bytes, var.fwd_states == nullptr);
    if (rc != LA_OK) return rc;
    return run_backward(Q, K, V, dO, dQ, dK, dV, lams, p, B, H, n, d, dt, (float *)workspace,
                        (hipStream_t)hip_stream, var);
}

// Caller-given layout: 16-byte granularity everywhere, rows at least d apart.
int check_layout(const la_layout *l, int d, LaLayout *out)
{
    if (!l) return LA_ERR_NULL;
    if (l->row_stride < d || l->batch_stride < 0 || l->head_stride < 0) return LA_ERR_SHAPE;
    if (l->row_stride % 8 || l->batch_stride % 8 || l->head_stride % 8) return LA_ERR_ALIGN;
    if (l->row_stride > INT32_MAX) return LA_ERR_SHAPE;
    out->bs = (long)l->batch_stride; out->hs = (long)l->head_stride; out->ld = (int)l->row_stride;
    return LA_OK;
}

// d_k = m * d_v: the scores add over the m slices of the query / key features, so the
// attention is the sum of m ordinary ones (App. A's kv state becomes m d_v x d_v states).
int check_wide(int dk, int dv)
{
    if (dv != 64 && dv != 128) return LA_ERR_SHAPE;
    if (dk < dv || dk % dv != 0 || dk / dv > 4) return LA_ERR_SHAPE;
    return LA_OK;
}

}  // namespace

extern "C" {

size_t la_workspace_bytes(int B, int H, int n, int d, la_dtype dt, int is_bwd)
{
    // backward: forward states of (V, K) and reverse states of (dO, Q) side by side
    if (check_common(B, H, n, d, dt) != LA_OK) return 0;
    return state_bytes(make_plan(B, H, n, d, dt), B, H, d) * (is_bwd ? 2 : 1);
}

int la_plan(int B, int H, int n, int d, la_dtype dt, int *tile, int *segment_len, int *segments)
{
    int rc = check_common(B, H, n, d, dt);
    if (rc != LA_OK) return rc;
    const Plan p = make_plan(B, H, n, d, dt);
    if (tile) *tile = p.tile;
    if (segment_len) *segment_len = p.L;
    if (segments) *segments = p.S;
    return LA_OK;
}

int la_fwd_state(const void *Q, const void *K, const void *V, const float *lambda, void *O,
                 const float *kv_in, float *kv_out,
                 int B, int H, int n, int d, la_dtype dt,
                 void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return forward(Q, K, V, lambda, O, kv_in, kv_out, B, H, n, d, dt, workspace, workspace_bytes,
                   hip_stream, Variant());
}

int la_fwd(const void *Q, const void *K, const void *V, const float *lambda, void *O,
           int B, int H, int n, int d, la_dtype dt,
           void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return forward(Q, K, V, lambda, O, nullptr, nullptr, B, H, n, d, dt, workspace, workspace_bytes,
                   hip_stream, Variant());
}

int la_fwd_static(const void *Q, const void *K, const void *V, const float *lambda, void *O,
                  int B, int H, int n, int d, la_dtype dt, void *hip_stream)
{
    int rc = check_common(B, H, n, d, dt);
    if (rc != LA_OK) return rc;
    const size_t need = state_bytes(make_plan(B, H, n, d, dt), B, H, d);
    if (need > (size_t)LA_STATIC_SCRATCH_BYTES) return LA_ERR_TOO_LARGE;
    void *scratch = nullptr;
    if (need > 0) {
        rc = static_scratch(&scratch);
        if (rc != LA_OK) return rc;
    }
    // Every state slot that is read is written earlier in the same call (pre-pass, then
    // segment scan), so what the previous call left in the scratch needs no clearing.
    return forward(Q, K, V, lambda, O, nullptr, nullptr, B, H, n, d, dt, scratch, need, hip_stream, Variant());
}

int la_fwd_swish(const void *Qp, const void *Kp, const void *V, const float *lambda, void *O,
                 int B, int H, int n, int d, la_dtype dt,
                 void *workspace, size_t workspace_bytes, void *hip_stream)
{
    // O = scan(phi(Qp), phi(Kp), V)
    Variant var;
    var.swish = true;
    return forward(Qp, Kp, V, lambda, O, nullptr, nullptr, B, H, n, d, dt, workspace, workspace_bytes,
                   hip_stream, var);
}

int la_fwd_strided(const void *Q, const void *K, const void *V, const float *lambda, void *O,
                   const la_layout *qkv_layout, const la_layout *o_layout,
                   int B, int H, int n, int d, la_dtype dt,
                   void *workspace, size_t workspace_bytes, void *hip_stream)
{
    LaLayout in, out;
    int rc = check_layout(qkv_layout, d, &in);
    if (rc == LA_OK) rc = check_layout(o_layout, d, &out);
    if (rc != LA_OK) return rc;
    Variant var;
    var.in = &in; var.out = &out;
    return forward(Q, K, V, lambda, O, nullptr, nullptr, B, H, n, d, dt, workspace, workspace_bytes,
                   hip_stream, var);
}

int la_fwd_wide(const void *Qw, const void *Kw, const void *V, const float *lambda, void *O,
                int B, int H, int n, int dk, int dv, la_dtype dt,
                void *workspace, size_t workspace_bytes, void *hip_stream)
{
    int rc = check_common(B, H, n, dv, dt);
    if (rc == LA_OK) rc = check_wide(dk, dv);
    if (rc != LA_OK) return rc;
    if (!Qw || !Kw) return LA_ERR_NULL;
    // d_k = 256, d_v = 128 in bf16, whole sequences: one kernel with the 256 x 128 state
    if (dt == LA_BF16 && dk == 256 && dv == 128 && make_plan(B, H, n, dv, dt).S == 1 &&
        !g_sw.wide_slices.load(std::memory_order_relaxed)) {
        if (!V || !O || !lambda) return LA_ERR_NULL;
        if (!aligned16(Qw) || !aligned16(Kw) || !aligned16(V) || !aligned16(O)) return LA_ERR_ALIGN;
        LaLambdas lams;
        rc = check_lambda(lambda, H, &lams);
        if (rc != LA_OK) return rc;
        Plan p = make_plan(B, H, n, dv, dt);
        ScanLaunch l = {};
        l.r[0] = make_args(Qw, Kw, V, O, p, H, n, dv, dt, nullptr, 0);
        l.nroles = 1; l.items = B * H;
        auto kern = la_scan_bf16_dma_wide;
        static std::once_flag once;
        static hipError_t attr_err = hipSuccess;
        std::call_once(once, [&] { attr_err = allow_lds(kern, DmaWideCfg::lds_bytes); });
        if (attr_err != hipSuccess) return LA_ERR_LAUNCH;
        hipLaunchKernelGGL(kern, dim3((unsigned)(B * H)), dim3(DmaWideCfg::NT), DmaWideCfg::lds_bytes,
                           (hipStream_t)hip_stream, l, lams);
        return hipGetLastError() == hipSuccess ? LA_OK : LA_ERR_LAUNCH;
    }
    const size_t esz = dt == LA_BF16 ? 2 : 4;
    for (int j = 0; j < dk / dv; ++j) {
        Variant var;
        var.wide_ld = dk;
        var.accumulate = j > 0;
        rc = forward((const char *)Qw + (size_t)j * dv * esz, (const char *)Kw + (size_t)j * dv * esz, V,
                     lambda, O, nullptr, nullptr, B, H, n, dv, dt, workspace, workspace_bytes, hip_stream, var);
        if (rc != LA_OK) return rc;
    }
    return LA_OK;
}

int la_decode_step(const void *q, const void *k, const void *v, const float *lambda,
                   float *kv, void *o, int B, int H, int d, la_dtype dt, void *hip_stream)
{
    int rc = check_common(B, H, 1, d, dt);
    if (rc != LA_OK) return rc;
    if (!q || !k || !v || !kv || !o || !lambda) return LA_ERR_NULL;
    if (!aligned16(kv) || ((uintptr_t)q & 3u) || ((uintptr_t)k & 3u) || ((uintptr_t)v & 3u) ||
        ((uintptr_t)o & 3u)) return LA_ERR_ALIGN;
    LaLambdas lams;
    rc = check_lambda(lambda, H, &lams);
    if (rc != LA_OK) return rc;
    hipStream_t s = (hipStream_t)hip_stream;
    dim3 grid((unsigned)((long)B * H)), block(256);
    if (dt == LA_BF16) {
        if (d == 64) hipLaunchKernelGGL((la_decode_kernel<64, true>), grid, block, 0, s, q, k, v, kv, o, H, lams);
        else hipLaunchKernelGGL((la_decode_kernel<128, true>), grid, block, 0, s, q, k, v, kv, o, H, lams);
    } else {
        if (d == 64) hipLaunchKernelGGL((la_decode_kernel<64, false>), grid, block, 0, s, q, k, v, kv, o, H, lams);
        else hipLaunchKernelGGL((la_decode_kernel<128, false>), grid, block, 0, s, q, k, v, kv, o, H, lams);
    }
    return hipGetLastError() == hipSuccess ? LA_OK : LA_ERR_LAUNCH;
}

int la_bwd(const void *Q, const void *K, const void *V, const float *lambda, const void *dO,
           void *dQ, void *dK, void *dV,
           int B, int H, int n, int d, la_dtype dt,
           void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return backward(Q, K, V, lambda, dO, dQ, dK, dV, B, H, n, d, dt, workspace, workspace_bytes,
                    hip_stream, Variant());
}

int la_bwd_saved(const void *Q, const void *K, const void *V, const float *lambda, const void *dO,
                 void *dQ, void *dK, void *dV, const void *fwd_workspace,
                 int B, int H, int n, int d, la_dtype dt,
                 void *workspace, size_t workspace_bytes, void *hip_stream)
{
    Variant var;
    if (la_workspace_bytes(B, H, n, d, dt, 0) > 0) {
        if (!fwd_workspace || ((uintptr_t)fwd_workspace & 255u)) return LA_ERR_WORKSPACE;
        var.fwd_states = (const float *)fwd_workspace;
    }
    return backward(Q, K, V, lambda, dO, dQ, dK, dV, B, H, n, d, dt, workspace, workspace_bytes,
                    hip_stream, var);
}

int la_bwd_swish(const void *Qp, const void *Kp, const void *V, const float *lambda, const void *dO,
                 void *dQp, void *dKp, void *dV,
                 int B, int H, int n, int d, la_dtype dt,
                 void *workspace, size_t workspace_bytes, void *hip_stream)
{
    Variant var;
    var.swish = true;
    return backward(Qp, Kp, V, lambda, dO, dQp, dKp, dV, B, H, n, d, dt, workspace, workspace_bytes,
                    hip_stream, var);
}

int la_bwd_strided(const void *Q, const void *K, const void *V, const float *lambda, const void *dO,
                   void *dQ, void *dK, void *dV,
                   const la_layout *qkv_layout, const la_layout *do_layout, const la_layout *grad_layout,
                   int B, int H, int n, int d, la_dtype dt,
                   void *workspace, size_t workspace_bytes, void *hip_stream)
{
    LaLayout in, dout, out;
    int rc = check_layout(qkv_layout, d, &in);
    if (rc == LA_OK) rc = check_layout(do_layout, d, &dout);
    if (rc == LA_OK) rc = check_layout(grad_layout, d, &out);
    if (rc != LA_OK) return rc;
    Variant var;
    var.in = &in; var.dout = &dout; var.out = &out;
    return backward(Q, K, V, lambda, dO, dQ, dK, dV, B, H, n, d, dt, workspace, workspace_bytes,
                    hip_stream, var);
}

int la_bwd_wide(const void *Qw, const void *Kw, const void *V, const float *lambda, const void *dO,
                void *dQw, void *dKw, void *dV,
                int B, int H, int n, int dk, int dv, la_dtype dt,
                void *workspace, size_t workspace_bytes, void *hip_stream)
{
    int rc = check_common(B, H, n, dv, dt);
    if (rc == LA_OK) rc = check_wide(dk, dv);
    if (rc != LA_OK) return rc;
    if (!Qw || !Kw || !dQw || !dKw) return LA_ERR_NULL;
    const size_t esz = dt == LA_BF16 ? 2 : 4;
    for (int j = 0; j < dk / dv; ++j) {
        Variant var;
        var.wide_ld = dk;
        var.accumulate = j > 0;
        const size_t off = (size_t)j * dv * esz;
        rc = backward((const char *)Qw + off, (const char *)Kw + off, V, lambda, dO, (char *)dQw + off,
                      (char *)dKw + off, dV, B, H, n, dv, dt, workspace, workspace_bytes, hip_stream, var);
        if (rc != LA_OK) return rc;
    }
    return LA_OK;
}

int la_gate_norm_fwd(const void *O, const void *U, void *Y, float eps,
                     int B, int H, int n, int d, la_dtype dt, void *hip_stream)
{
    int rc = check_common(B, H, n, d, dt);
    if (rc != LA_OK) return rc;
    if (B > 65535) return LA_ERR_SHAPE;
    if (!O || !U || !Y) return LA_ERR_NULL;
    if (!aligned16(O) || !aligned16(U) || !aligned16(Y)) return LA_ERR_ALIGN;
    if (!(eps >= 0.0f) || !std::isfinite(eps)) return LA_ERR_LAMBDA;
    GateArgs g;
    g.O = O; g.U = U; g.dY = nullptr; g.Y = Y; g.dO = nullptr; g.dU = nullptr;
    g.H = H; g.n = n; g.eps = eps;
    return run_gate_norm<false>(g, B, n, d, dt, (hipStream_t)hip_stream);
}

int la_gate_norm_bwd(const void *O, const void *U, const void *dY, void *dO, void *dU, float eps,
                     int B, int H, int n, int d, la_dtype dt, void *hip_stream)
{
    int rc = check_common(B, H, n, d, dt);
    if (rc != LA_OK) return rc;
    if (B > 65535) return LA_ERR_SHAPE;
    if (!O || !U || !dY || !dO || !dU) return LA_ERR_NULL;
    if (!aligned16(O) || !aligned16(U) || !aligned16(dY) || !aligned16(dO) || !aligned16(dU))
        return LA_ERR_ALIGN;
    if (!(eps >= 0.0f) || !std::isfinite(eps)) return LA_ERR_LAMBDA;
    GateArgs g;
    g.O = O; g.U = U; g.dY = dY; g.Y = nullptr; g.dO = dO; g.dU = dU;
    g.H = H; g.n = n; g.eps = eps;
    return run_gate_norm<true>(g, B, n, d, dt, (hipStream_t)hip_stream);
}

size_t la_lrpe_workspace_bytes(int B, int H, int n, int d)
{
    if (B < 1 || H < 1 || n < 1 || (d != 64 && d != 128)) return 0;
    const size_t tiles = ((size_t)n + LRPE_ROWS - 1) / LRPE_ROWS;
    return (size_t)B * H * tiles * d * sizeof(float);
}

int la_lrpe_rotate_fwd(const void *X, const float *theta, void *Xw,
                       int B, int H, int n, int d, la_dtype dt, void *hip_stream)
{
    int rc = check_common(B, H, n, d, dt);
    if (rc != LA_OK) return rc;
    if ((long)B * H > 65535) return LA_ERR_SHAPE;
    if (!X || !theta || !Xw) return LA_ERR_NULL;
    if (!aligned16(X) || !aligned16(Xw) || ((uintptr_t)theta & 3u)) return LA_ERR_ALIGN;
    LrpeArgs a;
    a.X = X; a.theta = theta; a.Xw = Xw; a.dX = nullptr; a.partial = nullptr;
    a.H = H; a.n = n; a.tiles = (n + LRPE_ROWS - 1) / LRPE_ROWS;
    return run_lrpe<false>(a, B, d, dt, (hipStream_t)hip_stream);
}

int la_lrpe_rotate_bwd(const void *X, const float *theta, const void *dXw, void *dX, float *dtheta,
                       int accumulate_dtheta, void *workspace, size_t workspace_bytes,
                       int B, int H, int n, int d, la_dtype dt, void *hip_stream)
{
    int rc = check_common(B, H, n, d, dt);
    if (rc != LA_OK) return rc;
    if ((long)B * H > 65535) return LA_ERR_SHAPE;
    if (!X || !theta || !dXw || !dX || !dtheta) return LA_ERR_NULL;
    if (!aligned16(X) || !aligned16(dXw) || !aligned16(dX) || ((uintptr_t)theta & 3u) ||
        ((uintptr_t)dtheta & 3u)) return LA_ERR_ALIGN;
    if (!workspace || ((uintptr_t)workspace & 255u) || workspace_bytes < la_lrpe_workspace_bytes(B, H, n, d))
        return LA_ERR_WORKSPACE;
    LrpeArgs a;
    a.X = X; a.theta = theta; a.Xw = const_cast<void *>(dXw); a.dX = dX; a.partial = (float *)workspace;
    a.H = H; a.n = n; a.tiles = (n + LRPE_ROWS - 1) / LRPE_ROWS;
    hipStream_t s = (hipStream_t)hip_stream;
    rc = run_lrpe<true>(a, B, d, dt, s);
    if (rc != LA_OK) return rc;
    hipLaunchKernelGGL(la_lrpe_theta_reduce, dim3((unsigned)(H * d / 32)), dim3(256), 0, s,
                       (const float *)workspace, dtheta, B, H, a.tiles, d, accumulate_dtheta ? 1 : 0);
    return hipGetLastError() == hipSuccess ? LA_OK : LA_ERR_LAUNCH;
}

const char *la_strerror(int status)
{
    switch (status) {
    case LA_OK: return "ok";
    case LA_ERR_NULL: return "a required pointer is NULL";
    case LA_ERR_SHAPE: return "invalid shape: need B,H,n >= 1, H <= 256, d in {64,128}";
    case LA_ERR_DTYPE: return "invalid dtype";
    case LA_ERR_LAMBDA: return "decay rate not finite or outside (0, 1] (or eps negative / not finite)";
    case LA_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case LA_ERR_LAUNCH: return "HIP kernel launch failed";
    case LA_ERR_ALIGN: return "tensor pointer not 16-byte aligned";
    case LA_ERR_TOO_LARGE: return "problem needs more scratch than the library's static buffer holds";
    default: return "unknown status";
    }
}

int la_profile_enable(int on)
{
    if (on) {
        while (g_prof.created < LA_PROFILE_MAX_LAUNCHES) {
            const int i = g_prof.created;
            if (hipEventCreate(&g_prof.start[i]) != hipSuccess) return LA_ERR_LAUNCH;
            if (hipEventCreate(&g_prof.stop[i]) != hipSuccess) {
                (void)hipEventDestroy(g_prof.start[i]);
                return LA_ERR_LAUNCH;
            }
            g_prof.created = i + 1;
        }
    }
    g_prof.on = on != 0;
    return LA_OK;
}

int la_debug_set(const char *name, long value)
{
    std::atomic<long> *sw = find_switch(name);
    if (!sw) return LA_ERR_NULL;
    sw->store(value, std::memory_order_relaxed);
    return LA_OK;
}

int la_debug_mfma_rate(int workgroups, int iters, float *sink, void *hip_stream)
{
    if (workgroups < 1 || iters < 1 || !sink) return LA_ERR_SHAPE;
    hipLaunchKernelGGL(la_mfma_rate_kernel, dim3((unsigned)workgroups), dim3(256), 0, (hipStream_t)hip_stream, sink, iters);
    return hipGetLastError() == hipSuccess ? LA_OK : LA_ERR_LAUNCH;
}

long la_debug_get(const char *name)
{
    std::atomic<long> *sw = find_switch(name);
    return sw ? sw->load(std::memory_order_relaxed) : -1;
}

int la_profile_collect(double *scan_kernel_ms, int *scan_kernel_launches)
{
    double total = 0.0;
    int ok = 0;
    for (int i = 0; i < g_prof.count; ++i) {
        if (hipEventSynchronize(g_prof.stop[i]) != hipSuccess) continue;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, g_prof.start[i], g_prof.stop[i]) == hipSuccess) {
            total += ms;
            ++ok;
        }
    }
    g_prof.count = 0;
    if (scan_kernel_ms) *scan_kernel_ms = total;
    if (scan_kernel_launches) *scan_kernel_launches = ok;
    return LA_OK;
}

}  // extern "C"
