// bf16 block scan fed by global -> LDS direct loads (gfx950), d = 128 and d = 64.  The text
// below describes d = 128 (256-byte tile rows, four waves); d = 64 is the same code with 128-byte
// rows, two waves per workgroup and its own chunk swizzle (DmaCfg, dma_swz).
//
// Same arithmetic as la_scan_bf16 (the block loop of Alg. 5 / Alg. 6: masked intra-block
// left product, inter-block right product against the running state, state update), same
// ownership (wave w owns value features [32w, 32w+32) of Out and of the state, which never
// leaves its accumulator registers), but the tiles take another road into the compute
// units, chosen so that more bytes are in flight per workgroup at no cost in registers:
//
//   * 32-row blocks.  A block's three tiles (A, Bm, C: 3 x 8 KB) are written into LDS by
//     global_load_lds_dwordx4, row-major and untouched, into one of three stages: the loads
//     of the next TWO blocks are outstanding while a block is computed, they occupy no
//     VGPRs and nobody executes a staging pass.
//   * Nothing is transposed or permuted on the way in.  Operands contracted over the
//     feature dim (scores, inter) are read as rows with ds_read_b128; operands contracted
//     over the token dim (C^T for the intra product, Bm^T and C for the state update) are
//     read from the same row-major tiles with the transposing ds_read_b64_tr_b16.
//   * The state feeds the inter product straight from the accumulators as before; instead
//     of storing the A tile with permuted columns, the two lane halves exchange the rows
//     of the state operand they lack with v_permlane32_swap.
//   * The masked scores P never touch LDS: every wave computes the whole 32 x 32 score
//     tile itself (8 MFMAs), and the accumulator layout of S^T is already the operand
//     layout of P^T, with the keys in the order (4g..4g+3, 8+4g..8+4g+3 per 16) that the
//     transposing reads of C^T are made to follow.
//   * The decay weights of the state update go onto the C fragments of the wave's own
//     slice (two fragments per block) rather than onto the whole Bm tile.
//   * Two barriers per block.  The four waves put their 32-feature slices of the Out tile
//     side by side in an 8 KB LDS area; after the second barrier each wave writes 8 whole
//     rows to memory, 1 KB contiguous per store instruction.  (Measured on the kernel's
//     load / store skeleton: whole rows instead of 64-byte pieces per wave are worth 5 to
//     10 %.)
//
// LDS tile layout: row r (0..31) at byte 256 r; its sixteen 16-byte chunks are stored at
// chunk position c ^ sw(r), sw(r) = the low four bits of r rotated left by two.  A direct
// load writes 64 lanes x 16 bytes to consecutive LDS addresses (4 rows); the swizzle is
// applied on the global side, lane -> chunk (lane & 15) ^ sw(row).  With it the 16 lanes
// of a ds_read_b128 group (16 rows, one chunk) cover sixteen different chunk positions, and
// the 32 lanes of half a transposing read (4 rows x 64 bytes) cover all sixteen positions
// twice over, once per 8-byte half: no bank is hit twice.  (With a rotation by one the
// transposing reads still collided in pairs: 7 % of the kernel's cycles.)
//
// ds_read_b64_tr_b16, as measured: in each group of 16 lanes, lane i receives, as its four
// 16-bit elements e = 0..3, element i % 4 of the 8 bytes that lane i / 4 + 4 e of the group
// points at.  With lane (a + 4 b) pointing at row b, columns 4a..4a+3, lane i ends up with
// column i of rows 0..3: a column-major fragment out of a row-major tile.
//
// The direct loads are issued from inline assembly and waited for by hand (s_waitcnt
// vmcnt(N), N = the 6 loads of the one block that may stay in flight plus the 2 stores of
// the block just finished), and the workgroup
// barrier is the bare s_barrier behind an LDS-only wait: the compiler, when it sees such a
// load, waits for ALL of them before the next transposing LDS read or fenced barrier, which
// would leave no prefetch at all.  Vector-memory instructions complete in issue order, so
// "at most the N youngest outstanding" means that everything older has landed; for that
// count to be exact every wave always issues both of its store instructions (rows past the
// end of the sequence re-store the last real row with the same data).
#pragma once
#include "la_kernels_bf16.h"

typedef __attribute__((address_space(3))) void la_lds_void;
typedef short la_s4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) la_s4 la_lds_s4;

// NS stages = NS - 1 blocks of prefetch.  NS = 3 lets two workgroups share a compute unit
// (80 KB each).  Measured: NS = 2 is as fast when 512 workgroups are resident and 4 % slower
// with 256; NS = 4 and 6 (one workgroup per compute unit) are 15 to 30 % slower: the path is
// not short of bytes in flight.
template <int NS_, int D_ = 128>
struct DmaCfg {
    static constexpr int D = D_, BK = 32;
    static constexpr int NS = NS_;
    static constexpr int NW = D / 32, NT = 64 * NW;          // one wave per 32 value features
    static constexpr int NTILE = 3;                          // tiles per stage: A, Bm, C
    static constexpr int PITCH = 2 * D;                      // bytes per tile row
    static constexpr int CPR = D / 8;                        // 16-byte chunks per row
    static constexpr int RPI = 64 / CPR;                     // rows one 64-lane load or store covers
    static constexpr int TILE_BYTES = BK * D * 2;            // 8192 at D = 128
    static constexpr int STAGE_BYTES = NTILE * TILE_BYTES;
    static constexpr int SO_BYTES = BK * D * 2;              // the Out tile, bf16
    static constexpr size_t lds_bytes = (size_t)NS * STAGE_BYTES + SO_BYTES;   // 81920 at NS = 3, D = 128
};

// Chunk swizzle of a tile row (see the layout note above).  D = 128: the low four bits of r
// rotated left by two.  D = 64 (128-byte rows, two rows per 256 bytes of banks): rows of equal
// parity among any sixteen get eight different values, and rows 4j .. 4j + 3 differ in bit 2
// between the two even and between the two odd ones, which is what the 16-row operand reads
// and the 4-row transposing reads need to touch every bank once.
template <int D>
__host__ __device__ constexpr int dma_swz(int r)
{
    if (D == 128) return ((r << 2) | ((r >> 2) & 3)) & 15;
    return ((((r & 3) ^ ((r >> 2) & 1)) << 1) | ((r >> 3) & 1)) & 7;
}
__device__ __forceinline__ int dma_sw(int r) { return dma_swz<128>(r); }

// wait until at most N vector-memory instructions of this wave are outstanding
template <int N>
__device__ __forceinline__ void la_wait_vm()
{
    static_assert(N >= 0 && N <= 63, "vmcnt is a 6-bit field");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
// ... at most n (a wave-uniform run-time value, n <= N): the count of the instruction is an
// immediate, so pick the largest even one that does not exceed n
template <int N>
__device__ __forceinline__ void la_wait_vm_le(int n)
{
    if constexpr (N <= 0) {
        la_wait_vm<0>();
    } else {
        if (n >= N) la_wait_vm<N>();
        else la_wait_vm_le<N - 2>(n);
    }
}
// LDS traffic of this wave complete, then the workgroup barrier; nothing moves across it
#define LA_LDS_BARRIER() asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory")

// One global -> LDS load of 16 bytes per lane: lane l's bytes land at lds_addr + 16 l
// (lds_addr wave-uniform, in M0).  NT: the non-temporal hint.
template <bool NT>
__device__ __forceinline__ void dma_load16(const void *gptr, uint32_t lds_addr)
{
    if (NT)
        asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off nt" ::"v"(gptr), "s"(lds_addr) : "memory", "m0");
    else
        asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gptr), "s"(lds_addr) : "memory", "m0");
}

__device__ __forceinline__ U2 lds_read_tr(const unsigned char *p)
{
    const la_s4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((la_lds_s4 *)p);
    return __builtin_bit_cast(U2, v);
}

// ABL != 0 builds measurement-only variants that leave parts of the work out (their results
// are wrong by design; reached only through the "ablate" debug switch):
//   1: no result stores   2: loads, waits and barriers only (no arithmetic, no stores)
//   3: arithmetic only (no loads, no stores; computes on whatever the LDS holds)
//   4: loads, barriers and result stores, no arithmetic (stores whatever the LDS area holds)
// NT_STORE: the result stores carry the non-temporal hint (a template parameter because
// two stores that differ only in the hint are merged into one plain store when they sit in
// the two arms of a run-time branch).
// TRIO: one launch holds the three scans of the backward pass, dQ forward in time and dK, dV
// reversed, the three workgroups of a (scan, segment) item side by side on one XCD; the direction is
// then a run-time property of the role and every tile load is cacheable (each tensor is read by two
// or three of the roles).  Measured against a dQ launch followed by a paired dK / dV launch: the
// kernel time is 3 % less (503 against 197 + 324 us under the profiler), a whole forward + backward
// step between level and 1.4 % faster depending on the box; what it saves is the boundary between
// two launches that each fill and drain the machine, and, while the tiles of the resident workgroups
// fit the Infinity Cache (sequences or segments of up to about 1024 tokens), a part of the reads
// that the forward and the reversed roles have in common.
// STRIDED: every operand has its own layout (ScanArgs::lA .. lO) instead of contiguous slabs.
template <bool REV_, bool NT_STORE, int ABL, int NS_, bool TRIO = false, bool STRIDED = false, int D_ = 128>
__global__ __launch_bounds__(2 * D_, NS_ <= 3 ? 2 : 1) void la_scan_bf16_dma(ScanLaunch launch, LaLambdas lams)
{
    using Cfg = DmaCfg<NS_, D_>;
    constexpr int D = Cfg::D, BK = Cfg::BK, NS = Cfg::NS, NTILE = Cfg::NTILE;
    constexpr int PITCH = Cfg::PITCH, CPR = Cfg::CPR, RPI = Cfg::RPI;
    constexpr int SW8 = dma_swz<D>(8);         // swizzle of row r + 8 = swizzle of row r ^ SW8
    constexpr int KS_D = D / 16;               // k-steps over the feature dim (8)
    constexpr int KS_B = BK / 16;              // k-steps over the block rows (2)
    constexpr int MT_D = D / 32;               // 32-row tiles over the feature dim (4)
    constexpr int SPW = (BK / RPI) / Cfg::NW;  // load slots (RPI rows each) per wave and tile: 2
    constexpr int LOADS = NTILE * SPW;         // direct loads per wave and block

    extern __shared__ __align__(16) unsigned char smem_dma[];

    const int tid = threadIdx.x;
    const int l = tid & 63, l32 = l & 31, g = l >> 5;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);      // wave index = value-feature slice, in a scalar register

    int item = blockIdx.x, role = 0;
    if (TRIO) {
        const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
        role = slot % 3;
        item = (slot / 3) * 8 + xcd;
        if (item >= launch.items) return;
    } else if (launch.nroles == 2) {
        const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
        role = slot & 1;
        item = (slot >> 1) * 8 + xcd;
        if (item >= launch.items) return;
    }
    const bool REV = TRIO ? (role != 0) : REV_;
    const ScanArgs &a = launch.r[role];
    // Consecutive items are the segments of one scan, except for token-major tensors (STRIDED
    // with the heads of a token side by side in memory, head stride < row stride): there they
    // are the scans of one segment, so that workgroups dispatched together, on different XCDs,
    // read neighbouring pieces of the same rows.  Measured on [1, 65536, 16, 128]: la_bwd 0.65
    // instead of 0.75 ms; contiguous slabs are a little slower in that order.
    const bool seg_major = STRIDED && a.lA.hs < (long)a.lA.ld;
    const int nscans = launch.items / a.S;
    const int seg = seg_major ? item / nscans : item % a.S;
    const int scan = seg_major ? item % nscans : item / a.S;
    const float lg = lams.lg2[scan % a.H];
    auto pw = [lg](int k) -> float { return exp2f((float)k * lg); };

    const int seg_lo = seg * a.L;
    const int seg_hi = min(a.n, seg_lo + a.L);
    const int nblk = (seg_hi - seg_lo + BK - 1) / BK;

    // tiles of a stage, in LDS order: A, Bm, C.  STRIDED: every operand has its own layout (slab
    // offsets per batch and head, rows ld elements apart); else contiguous [scans, n, D].
    const uint16_t *gT[NTILE];
    uint16_t *gO;
    int ldT[NTILE], ldO;
    if (STRIDED) {
        const long bb = scan / a.H, hh = scan % a.H;
        gT[0] = (const uint16_t *)a.A + bb * a.lA.bs + hh * a.lA.hs;
        gT[1] = (const uint16_t *)a.Bm + bb * a.lB.bs + hh * a.lB.hs;
        gT[2] = (const uint16_t *)a.C + bb * a.lC.bs + hh * a.lC.hs;
        gO = (uint16_t *)a.Out + bb * a.lO.bs + hh * a.lO.hs;
        ldT[0] = a.lA.ld; ldT[1] = a.lB.ld; ldT[2] = a.lC.ld; ldO = a.lO.ld;
    } else {
        const size_t base = (size_t)scan * a.n * D;
        gT[0] = (const uint16_t *)a.A + base;
        gT[1] = (const uint16_t *)a.Bm + base;
        gT[2] = (const uint16_t *)a.C + base;
        gO = (uint16_t *)a.Out + base;
        ldT[0] = ldT[1] = ldT[2] = ldO = D;
    }

    // ---- per-lane constants ----------------------------------------------------------
    // key / token held in slot e (0..7) of k-step ks: 16 ks + (e < 4 ? 4g + e : 8 + 4g + e - 4);
    // the same order as accumulator register v = 8 ks + e of a 32 x 32 tile (row 8 (v/4) + 4g + v%4)
    float mk[16];                              // decay mask of the score tile: lane = q, register = key
    float wt[16];                              // state-update weight of the token in slot (ks, e)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int key = 8 * (v >> 2) + 4 * g + (v & 3);
        const int dist = REV ? (key - l32) : (l32 - key);
        mk[v] = dist >= 0 ? pw(dist) : 0.0f;
        wt[v] = REV ? pw(key) : pw(BK - 1 - key);
    }
    const float rsq = REV ? pw(BK - l32) : pw(l32 + 1);          // inter-block scale of column q = l32
    float lamBK = pw(BK);
    const bool want_final = !REV && a.st_out != nullptr && seg == a.S - 1;

    // row-operand reads: row l32, chunk 2 ks + g
    const int ro_base = l32 * PITCH;
    const int ro_sw = dma_swz<D>(l32) ^ g;                       // chunk position = (2 ks) ^ ro_sw
    // transposing reads: lane = (a4 + 4 b4) + 16 h16 + 32 g
    const int a4 = l & 3, b4 = (l >> 2) & 3, h16 = (l >> 4) & 1;
    const int tr_base = (4 * g + b4) * PITCH + 8 * (a4 & 1);     // row 4g + b4, 8-byte half of the chunk
    const int tr_sw = (2 * h16 + (a4 >> 1)) ^ dma_swz<D>(4 * g + b4);   // chunk within the 32 columns ^ sw(row), sel = 0
    // direct loads: load slot ii = SPW w + j covers tile rows 4 ii .. 4 ii + 3
    int dma_row[SPW], dma_col[SPW];
#pragma unroll
    for (int j = 0; j < SPW; ++j) {
        dma_row[j] = RPI * (SPW * w + j) + l / CPR;
        dma_col[j] = 8 * ((l % CPR) ^ dma_swz<D>(dma_row[j]));   // element offset of the chunk fetched
    }
    // Out tile: row q at 256 q, chunk c (8 features) at position c ^ (q & 15)
    unsigned char *sO = smem_dma + NS * Cfg::STAGE_BYTES;
    // LDS byte address of the first stage, as the direct loads want it (wave-uniform)
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(la_lds_void *)smem_dma);

    // ---- running state: St[i][j], j in this wave's slice ------------------------------
    f32x16_t st[MT_D];
    const float *gSt = la_entering_state(a, scan, seg, REV, lg, D * D);
    const bool has_init = gSt != nullptr;
    if (has_init && a.transpose_init) {
        // the stored state is that of the scan with Bm and C exchanged: through LDS, transposed
        float *sT = reinterpret_cast<float *>(smem_dma);         // [D][D+1]
        for (int e = tid * 4; e < D * D; e += 4 * Cfg::NT) {
            const float4 x = *(const float4 *)(gSt + e);
            float *q = sT + (e / D) * (D + 1) + (e % D);
            q[0] = x.x; q[1] = x.y; q[2] = x.z; q[3] = x.w;
        }
        __syncthreads();
#pragma unroll
        for (int mt = 0; mt < MT_D; ++mt)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int i = 32 * mt + 8 * (v >> 2) + 4 * g + (v & 3);
                st[mt][v] = sT[(32 * w + l32) * (D + 1) + i];
            }
        __syncthreads();
    } else {
#pragma unroll
        for (int mt = 0; mt < MT_D; ++mt)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int i = 32 * mt + 8 * (v >> 2) + 4 * g + (v & 3);
                st[mt][v] = has_init ? gSt[(size_t)i * D + 32 * w + l32] : 0.0f;
            }
    }

    // ---- global -> LDS loads of one block ------------------------------------------------
    // Rows past the segment end fetch the segment's last row (always in bounds) and are
    // zeroed in LDS by the lane that fetched them once the load has landed.
    // Tiles that no other workgroup reads carry the non-temporal hint: everything in a
    // single-scan launch, the A operand in a paired launch.
    const bool nt_all = launch.nroles == 1;
    const bool nt_a = !TRIO;                    // the A operand is private to a scan except in a trio
    const auto blk_of = [&](int ib) { return REV ? (nblk - 1 - ib) : ib; };
    auto issue = [&](int ib, int stage) {
        if (ABL == 3) return;
        const int t0 = seg_lo + blk_of(ib) * BK;
#pragma unroll
        for (int j = 0; j < SPW; ++j) {
            const size_t row = (size_t)min(t0 + dma_row[j], seg_hi - 1);
            const uint32_t dst = lds0 + stage * Cfg::STAGE_BYTES + (SPW * w + j) * 1024;   // lane l lands at + 16 l
            if (nt_a) dma_load16<true>(gT[0] + row * ldT[0] + dma_col[j], dst);
            else dma_load16<false>(gT[0] + row * ldT[0] + dma_col[j], dst);
            if (nt_all) {
#pragma unroll
                for (int t = 1; t < NTILE; ++t)
                    dma_load16<true>(gT[t] + row * ldT[t] + dma_col[j], dst + t * Cfg::TILE_BYTES);
            } else {
#pragma unroll
                for (int t = 1; t < NTILE; ++t)
                    dma_load16<false>(gT[t] + row * ldT[t] + dma_col[j], dst + t * Cfg::TILE_BYTES);
            }
        }
    };
    // ---- Out tile: LDS -> memory, 8 whole rows per wave.  Always two store instructions
    // with every lane active (see the note on counting above): a row past the end of the
    // sequence stores the last real row again.
    auto store_out = [&](int t0) {
        if (ABL != 0 && ABL != 4) return;
        const int last = min(BK, seg_hi - t0) - 1;
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            const int row = min(2 * RPI * w + RPI * p + l / CPR, last), ch = l % CPR;
            const U4 o = *(const U4 *)(sO + row * PITCH + ((ch ^ (row & (CPR - 1))) << 4));
            U4 *dst = (U4 *)(gO + (size_t)(t0 + row) * ldO + 8 * ch);
            if (NT_STORE) __builtin_nontemporal_store(o, dst);
            else *dst = o;
        }
    };

    constexpr int PF = NS - 1;                 // blocks of prefetch
#pragma unroll
    for (int i = 0; i < PF; ++i)
        if (i < nblk) issue(i, i);
    constexpr int ST = (ABL == 0 || ABL == 4) ? 2 : 0;           // store instructions per wave and block

    int stage = 0;
    for (int ib = 0; ib < nblk; ++ib) {
        const int t0 = seg_lo + blk_of(ib) * BK;
        unsigned char *sb = smem_dma + stage * Cfg::STAGE_BYTES;
        // Every iteration issues the loads of block ib + PF, then (at its end) the 2 stores of
        // block ib.  Counting back from the youngest instruction, what may still be outstanding
        // when block ib must have landed: the stores of the last PF - 1 blocks and the loads of
        // blocks ib + 1 .. ib + PF - 1, as far as they exist (at the start the first PF blocks
        // were issued back to back, with fewer stores among them; near the end some loads were
        // never issued).  Short segments simply wait for everything.
        if (nblk < 2 * PF + 1 || ib + 1 >= nblk) {
            la_wait_vm<0>();
        } else {
            const int young = min(PF - 1, nblk - 1 - ib);    // blocks whose loads are younger
            const int olds = min(PF - 1, ib);                // blocks whose stores are younger
            la_wait_vm_le<(PF - 1) * (LOADS + ST)>(LOADS * young + ST * olds);
        }
        if (t0 + BK > seg_hi) {                 // partial block: zero padding (exact)
            const U4 z = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int j = 0; j < SPW; ++j)
                if (t0 + dma_row[j] >= seg_hi) {
                    unsigned char *dst = sb + (SPW * w + j) * 1024 + 16 * l;
#pragma unroll
                    for (int t = 0; t < NTILE; ++t) *(U4 *)(dst + t * Cfg::TILE_BYTES) = z;
                }
            if (want_final) {
                // The state handed back must be the one after the last real token: weight
                // row r of the m real rows by lambda^(m-1-r) and decay the old state by
                // lambda^m instead of padding the block out to BK rows.
                const int m = seg_hi - t0;
#pragma unroll
                for (int v = 0; v < 16; ++v) wt[v] = pw(max(m - 1 - (8 * (v >> 2) + 4 * g + (v & 3)), 0));
                lamBK = pw(m);
            }
        }
        LA_LDS_BARRIER();                       // the block has landed for every wave; the stage
                                                // of block ib - 1 is free for block ib + PF
        if (ib + PF < nblk) issue(ib + PF, stage >= 1 ? stage - 1 : NS - 1);

        if (ABL == 2 || ABL == 4) {
            if (ABL == 4) {
                LA_LDS_BARRIER();
                store_out(t0);
            }
            stage = stage + 1 < NS ? stage + 1 : 0;
            continue;
        }
        const unsigned char *sA = sb, *sB = sb + Cfg::TILE_BYTES, *sC = sb + 2 * Cfg::TILE_BYTES;

        // ---- row fragments of A (both products) and of Bm (scores) ---------------------
        U4 fa[KS_D];
#pragma unroll
        for (int ks = 0; ks < KS_D; ++ks) fa[ks] = *(const U4 *)(sA + ro_base + (((2 * ks) ^ ro_sw) << 4));
        // ---- scores: S^T = Bm A^T (lane = q, registers = keys), in two halves of the k range
        f32x16_t s = {0};
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            U4 fb[KS_D / 2];
#pragma unroll
            for (int k = 0; k < KS_D / 2; ++k)
                fb[k] = *(const U4 *)(sB + ro_base + (((2 * (KS_D / 2 * h + k)) ^ ro_sw) << 4));
            LA_BATCH_FENCE();
#pragma unroll
            for (int k = 0; k < KS_D / 2; ++k) s = mfma32(fb[k], fa[KS_D / 2 * h + k], s);
        }
        // ---- inter block: x^T = St^T A^T; the state operand is made from the accumulators:
        // lane half g holds rows 4g..4g+3 and 8+4g..8+4g+3 of every 16, the operand wants
        // rows 8g..8g+7: the halves exchange what they lack.
        f32x16_t x = {0};
#pragma unroll
        for (int ks = 0; ks < KS_D; ++ks) {
            const int mt = ks >> 1, h8 = 8 * (ks & 1);
            const uint32_t x0 = pack2_bf16(st[mt][h8 + 0], st[mt][h8 + 1]);
            const uint32_t x1 = pack2_bf16(st[mt][h8 + 2], st[mt][h8 + 3]);
            const uint32_t y0 = pack2_bf16(st[mt][h8 + 4], st[mt][h8 + 5]);
            const uint32_t y1 = pack2_bf16(st[mt][h8 + 6], st[mt][h8 + 7]);
            const auto s0 = __builtin_amdgcn_permlane32_swap(x0, y0, false, false);
            const auto s1 = __builtin_amdgcn_permlane32_swap(x1, y1, false, false);
            const U4 so = {s0[0], s1[0], s0[1], s1[1]};
            x = mfma32(so, fa[ks], x);
        }
        // ---- C^T fragments of this wave's slice (transposing reads), plain and weighted ---
        U4 cf[KS_B], cw[KS_B];
#pragma unroll
        for (int ks = 0; ks < KS_B; ++ks) {
            const unsigned char *p = sC + tr_base + 16 * ks * PITCH;
            const U2 lo = lds_read_tr(p + ((((4 * w) ^ tr_sw)) << 4));
            const U2 hi = lds_read_tr(p + 8 * PITCH + ((((4 * w) ^ tr_sw ^ SW8)) << 4));
            cf[ks] = U4{lo[0], lo[1], hi[0], hi[1]};
        }
        // ---- P = bf16(S * mask) stays in registers: it is already the operand of the intra product
        U4 pk[KS_B];
#pragma unroll
        for (int ks = 0; ks < KS_B; ++ks)
#pragma unroll
            for (int e = 0; e < 4; ++e)
                pk[ks][e] = pack2_bf16(s[8 * ks + 2 * e] * mk[8 * ks + 2 * e],
                                       s[8 * ks + 2 * e + 1] * mk[8 * ks + 2 * e + 1]);
#pragma unroll
        for (int v = 0; v < 16; ++v) x[v] *= rsq;
        // ---- intra block: Out^T += C^T P^T
#pragma unroll
        for (int ks = 0; ks < KS_B; ++ks) x = mfma32(cf[ks], pk[ks], x);
        // ---- Out tile -> LDS (bf16): lane holds 4 consecutive features per v4
#pragma unroll
        for (int v4 = 0; v4 < 4; ++v4) {
            U2 o;
            o[0] = pack2_bf16(x[4 * v4 + 0], x[4 * v4 + 1]);
            o[1] = pack2_bf16(x[4 * v4 + 2], x[4 * v4 + 3]);
            *(U2 *)(sO + l32 * PITCH + (((4 * w + v4) ^ (l32 & (CPR - 1))) << 4) + 8 * g) = o;
        }
#pragma unroll
        for (int ks = 0; ks < KS_B; ++ks)
#pragma unroll
            for (int e = 0; e < 4; ++e)
                cw[ks][e] = pack2_bf16(bf16_lo(cf[ks][e]) * wt[8 * ks + 2 * e],
                                       bf16_hi(cf[ks][e]) * wt[8 * ks + 2 * e + 1]);
        // ---- state update: St = lambda^BK St + Bm^T (w C) -----------------------------------
#pragma unroll
        for (int mt = 0; mt < MT_D; ++mt) {
            U4 bt[KS_B];
#pragma unroll
            for (int ks = 0; ks < KS_B; ++ks) {
                const unsigned char *p = sB + tr_base + 16 * ks * PITCH;
                const U2 lo = lds_read_tr(p + ((((4 * mt) ^ tr_sw)) << 4));
                const U2 hi = lds_read_tr(p + 8 * PITCH + ((((4 * mt) ^ tr_sw ^ SW8)) << 4));
                bt[ks] = U4{lo[0], lo[1], hi[0], hi[1]};
            }
            LA_BATCH_FENCE();
            f32x16_t u = st[mt];
#pragma unroll
            for (int v = 0; v < 16; ++v) u[v] *= lamBK;
#pragma unroll
            for (int ks = 0; ks < KS_B; ++ks) u = mfma32(bt[ks], cw[ks], u);
            st[mt] = u;
        }
        LA_LDS_BARRIER();                       // the Out tile is complete
        store_out(t0);
        stage = stage + 1 < NS ? stage + 1 : 0;
    }
    if (ABL != 0) {                             // keep the arithmetic alive: one store per wave
        float keep = 0.f;
#pragma unroll
        for (int mt = 0; mt < MT_D; ++mt) keep += st[mt][0];
        if (l == 0) gO[(size_t)seg_lo * ldO + 32 * w] = (uint16_t)(__float_as_uint(keep + (float)sO[l]) >> 16);
    }

    if (want_final) {
        float *dst = a.st_out + (size_t)scan * (D * D);
#pragma unroll
        for (int mt = 0; mt < MT_D; ++mt)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int i = 32 * mt + 8 * (v >> 2) + 4 * g + (v & 3);
                dst[(size_t)i * D + 32 * w + l32] = st[mt][v];
            }
    }
}

// ---- segment-state pre-pass on the same machinery --------------------------------------
// The local end state of every segment (see la_kernels_prepass.h for what it is and how the
// launch is laid out: roles, head order, decay cut-off), computed as the state update of the
// block scan alone: per 32-row block the Bm and C tiles arrive by direct loads (2 x 8 KB per
// stage), Bm^T and this wave's C fragments come from the transposing reads, and the decay is
// folded into the weights put on the C fragments (row r of block k is weighted by its full
// distance to the segment's far end), so the accumulator is never rescaled and partial sums
// over any subset of the blocks simply add.
//
// That last property is what the workgroup layout uses.  A segment's blocks form one
// dependent chain (wait for the block, barrier, issue the next load, 20 LDS reads, 8 MFMAs),
// and a slowly decaying head must read all 64 blocks of a 2048-token segment while the quickly
// decaying heads are long done.  A workgroup is therefore G = 4 groups of four waves; group q
// takes blocks q, q + 4, ... with its own two LDS stages and its own accumulators, and at the
// end the groups' partial states are added through LDS in a fixed order (group 0 + 1 + 2 + 3:
// deterministic).  The chain is a quarter as long and four of them overlap on one compute
// unit; neither the workspace nor any other kernel knows about it.  Measured at 16 heads x
// 64K tokens (32 segments a head), la_fwd / la_bwd in ms: one group with two stages 0.285 /
// 0.612, two groups 0.267 / 0.600, four groups 0.261 / 0.604; one group with five stages
// (four blocks of prefetch, the earlier layout) 0.266 / 0.62.  All but the first sit at about
// 45 us per launch of 512 workgroups, i.e. the kernel's 224 MB at 5 TB/s: the pre-pass is
// bound by its bytes and by the ramp of a short launch, not by the chain, once either the
// prefetch is deep enough or the chain is split.
template <int G_, int D_ = 128>
struct DmaPrepassCfg {
    static constexpr int D = D_, BK = 32, NS = 2, G = G_, NW = D / 32, NT = 64 * NW * G_;
    static constexpr int PITCH = 2 * D, CPR = D / 8, RPI = 64 / CPR;
    static constexpr int TILE_BYTES = BK * D * 2;
    static constexpr int STAGE_BYTES = 2 * TILE_BYTES;       // Bm, C
    static constexpr size_t raw_bytes = (size_t)G * NS * STAGE_BYTES;
    // the partial states are exchanged through a [D / 2][64 NW] fp32 area laid over the stages
    static constexpr size_t xchg_bytes = (size_t)(D / 2) * 64 * NW * 4;
    static constexpr size_t lds_bytes = raw_bytes > xchg_bytes ? raw_bytes : xchg_bytes;
};

template <int G_, bool STRIDED = false, int D_ = 128>
__global__ __launch_bounds__(2 * D_ * G_, 1) void la_prepass_bf16_dma(ScanLaunch launch, LaLambdas lams)
{
    using Cfg = DmaPrepassCfg<G_, D_>;
    constexpr int D = Cfg::D, BK = Cfg::BK, NS = Cfg::NS, G = Cfg::G, NW = Cfg::NW;
    constexpr int PITCH = Cfg::PITCH, CPR = Cfg::CPR, RPI = Cfg::RPI;
    constexpr int SW8 = dma_swz<D>(8);
    constexpr int KS_B = BK / 16, MT_D = D / 32;

    extern __shared__ __align__(16) unsigned char smem_dma[];

    const int tid = threadIdx.x;
    const int l = tid & 63, l32 = l & 31, g = l >> 5;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int w = wv % NW;                                   // value-feature slice of this wave
    const int gq = wv / NW;                                  // group: blocks gq, gq + G, ...

    const int role = launch.nroles == 2 ? (int)(blockIdx.x / launch.items) : 0;
    const int item = launch.nroles == 2 ? (int)(blockIdx.x % launch.items) : (int)blockIdx.x;
    const ScanArgs &a = launch.r[role];
    const int seg = item % a.S;
    const int bh = item / a.S;                               // (head in dispatch order, batch)
    const int scan = (bh % a.B) * a.H + lams.order[bh / a.B];
    const bool rev = a.rev != 0;
    if (!rev && seg == a.S - 1) return;                      // never consumed
    if (rev && seg == 0) return;

    const float lg = lams.lg2[scan % a.H];
    auto pw = [lg](int k) -> float { return exp2f((float)k * lg); };

    const int seg_lo = seg * a.L;
    const int seg_hi = min(a.n, seg_lo + a.L);
    const int nblk = (seg_hi - seg_lo + BK - 1) / BK;
    int ib0 = 0;                                             // decay cut-off
    if (a.skip_bits > 0.f && lg < 0.f) {
        const float reach = a.skip_bits / -lg;
        if (reach < (float)(nblk * BK)) ib0 = max(0, nblk - ((int)(reach / BK) + 2));
    }
    const int rounds = (nblk - ib0 + G - 1) / G;             // iterations, the same for every group

    const uint16_t *gB, *gC;
    int ldB, ldC;
    if (STRIDED) {
        const long bb = scan / a.H, hh = scan % a.H;
        gB = (const uint16_t *)a.Bm + bb * a.lB.bs + hh * a.lB.hs;
        gC = (const uint16_t *)a.C + bb * a.lC.bs + hh * a.lC.hs;
        ldB = a.lB.ld; ldC = a.lC.ld;
    } else {
        const size_t base = (size_t)scan * a.n * D;
        gB = (const uint16_t *)a.Bm + base;
        gC = (const uint16_t *)a.C + base;
        ldB = ldC = D;
    }
    float *gSt = a.states + ((size_t)scan * a.S + seg) * (size_t)(D * D);

    float wt[16];                              // weight of the token in slot (ks, e) inside a block
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int key = 8 * (v >> 2) + 4 * g + (v & 3);
        wt[v] = rev ? pw(key) : pw(BK - 1 - key);
    }
    const int a4 = l & 3, b4 = (l >> 2) & 3, h16 = (l >> 4) & 1;
    const int tr_base = (4 * g + b4) * PITCH + 8 * (a4 & 1);
    const int tr_sw = (2 * h16 + (a4 >> 1)) ^ dma_swz<D>(4 * g + b4);
    int dma_row[2], dma_col[2];                              // (BK / RPI) / NW = 2 load slots per wave and tile
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        dma_row[j] = RPI * (2 * w + j) + l / CPR;
        dma_col[j] = 8 * ((l % CPR) ^ dma_swz<D>(dma_row[j]));
    }
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(la_lds_void *)smem_dma);
    const int group_off = gq * NS * Cfg::STAGE_BYTES;

    f32x16_t st[MT_D];
#pragma unroll
    for (int mt = 0; mt < MT_D; ++mt)
#pragma unroll
        for (int v = 0; v < 16; ++v) st[mt][v] = 0.0f;

    const auto blk_of = [&](int ib) { return rev ? (nblk - 1 - ib) : ib; };
    auto issue = [&](int ib, int stage) {
        const int t0 = seg_lo + blk_of(ib) * BK;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const size_t row = (size_t)min(t0 + dma_row[j], seg_hi - 1);
            const uint32_t dst = lds0 + group_off + stage * Cfg::STAGE_BYTES + (2 * w + j) * 1024;
            dma_load16<true>(gB + row * ldB + dma_col[j], dst);
            dma_load16<true>(gC + row * ldC + dma_col[j], dst + Cfg::TILE_BYTES);
        }
    };

    if (ib0 + gq < nblk) issue(ib0 + gq, 0);

    for (int it = 0; it < rounds; ++it) {
        const int ib = ib0 + gq + it * G;
        const bool live = ib < nblk;
        const int stage = it & 1;
        unsigned char *sb = smem_dma + group_off + stage * Cfg::STAGE_BYTES;
        const int blk = blk_of(live ? ib : ib0);
        const int t0 = seg_lo + blk * BK;
        la_wait_vm<0>();                        // this group's only outstanding loads are this block's
        if (live && t0 + BK > seg_hi) {         // partial block: zero padding (exact)
            const U4 z = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int j = 0; j < 2; ++j)
                if (t0 + dma_row[j] >= seg_hi) {
                    unsigned char *dst = sb + (2 * w + j) * 1024 + 16 * l;
                    *(U4 *)dst = z;
                    *(U4 *)(dst + Cfg::TILE_BYTES) = z;
                }
        }
        LA_LDS_BARRIER();                       // landed for every wave; the other stage is free
        if (ib + G < nblk) issue(ib + G, stage ^ 1);
        if (!live) continue;

        const unsigned char *sB = sb, *sC = sb + Cfg::TILE_BYTES;
        // distance of this block to the segment's far end, folded into the weights
        const float mu = rev ? pw(blk * BK) : pw((nblk - 1 - blk) * BK);
        // the LDS reads go out in batches (one of 20 reads; at four groups, where a wave has a
        // quarter of the registers, two of 12 and 8), each followed by its MFMAs: independent
        // accumulator chains, interleaved
        constexpr int MB = (G == 4 && MT_D > 2) ? 2 : MT_D;
        U2 rc[KS_B][2];
        U4 cw[KS_B];
#pragma unroll
        for (int m0 = 0; m0 < MT_D; m0 += MB) {
            U2 rb[MB][KS_B][2];
            if (m0 == 0) {
#pragma unroll
                for (int ks = 0; ks < KS_B; ++ks) {
                    const unsigned char *p = sC + tr_base + 16 * ks * PITCH;
                    rc[ks][0] = lds_read_tr(p + ((((4 * w) ^ tr_sw)) << 4));
                    rc[ks][1] = lds_read_tr(p + 8 * PITCH + ((((4 * w) ^ tr_sw ^ SW8)) << 4));
                }
            }
#pragma unroll
            for (int m = 0; m < MB; ++m)
#pragma unroll
                for (int ks = 0; ks < KS_B; ++ks) {
                    const unsigned char *p = sB + tr_base + 16 * ks * PITCH;
                    rb[m][ks][0] = lds_read_tr(p + ((((4 * (m0 + m)) ^ tr_sw)) << 4));
                    rb[m][ks][1] = lds_read_tr(p + 8 * PITCH + ((((4 * (m0 + m)) ^ tr_sw ^ SW8)) << 4));
                }
            LA_BATCH_FENCE();
            if (m0 == 0) {
#pragma unroll
                for (int ks = 0; ks < KS_B; ++ks) {
                    const U4 cf = {rc[ks][0][0], rc[ks][0][1], rc[ks][1][0], rc[ks][1][1]};
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        cw[ks][e] = pack2_bf16(bf16_lo(cf[e]) * (wt[8 * ks + 2 * e] * mu),
                                               bf16_hi(cf[e]) * (wt[8 * ks + 2 * e + 1] * mu));
                }
            }
#pragma unroll
            for (int ks = 0; ks < KS_B; ++ks)
#pragma unroll
                for (int m = 0; m < MB; ++m) {
                    const U4 bt = {rb[m][ks][0][0], rb[m][ks][0][1], rb[m][ks][1][0], rb[m][ks][1][1]};
                    st[m0 + m] = mfma32(bt, cw[ks], st[m0 + m]);
                }
        }
    }

    // ---- the groups' partial states, added in a fixed order through LDS ------------------
    if (G > 1) {
        float *sX = reinterpret_cast<float *>(smem_dma);     // [16 MT_D][64 NW]: entry (mt, v) of thread (w, l)
        LA_LDS_BARRIER();                       // every group is done with its stages
#pragma unroll 1
        for (int r = 1; r < G; ++r) {
            if (gq == r) {
#pragma unroll
                for (int mt = 0; mt < MT_D; ++mt)
#pragma unroll
                    for (int v = 0; v < 16; ++v) sX[(16 * mt + v) * (64 * NW) + 64 * w + l] = st[mt][v];
            }
            LA_LDS_BARRIER();
            if (gq == 0) {
#pragma unroll
                for (int mt = 0; mt < MT_D; ++mt)
#pragma unroll
                    for (int v = 0; v < 16; ++v) st[mt][v] += sX[(16 * mt + v) * (64 * NW) + 64 * w + l];
            }
            LA_LDS_BARRIER();
        }
        if (gq != 0) return;
    }

#pragma unroll
    for (int mt = 0; mt < MT_D; ++mt)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int i = 32 * mt + 8 * (v >> 2) + 4 * g + (v & 3);
            gSt[(size_t)i * D + 32 * w + l32] = st[mt][v];
        }
}
