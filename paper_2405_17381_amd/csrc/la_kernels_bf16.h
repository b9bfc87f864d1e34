// bf16 path: the block loop of Alg. 5 / Alg. 6 on gfx950 matrix cores.
// (The segment-state pre-pass that lets one scan be cut into segments is in
// la_kernels_prepass.h and reuses the tile layouts and helpers defined here.)
//
// One workgroup of D/32 wavefronts walks the blocks (BK = 64 rows) of one
// segment of one (batch, head) scan.  All four contractions of a block run on
// v_mfma_f32_32x32x16_bf16 with fp32 accumulation:
//
//   S^T   = Bm A^T              scores, transposed; contraction over the feature dim
//   Out^T = C^T P^T             intra block, P = bf16(S * decay mask)
//   Out^T+= (St^T A^T) * scale  inter block, against the running state
//   St    = lambda^BK St + (w * Bm)^T C
//
// Ownership.  Wave w owns the value-feature slice j in [32w, 32w+32): its
// columns of Out and of the state St[:, slice].  The state never leaves the
// wave's accumulator registers: the fp32 accumulator layout of a 32x32 tile
// (lane = column j, registers = rows i) is exactly an MFMA operand with a
// permuted contraction order, so it is rounded to bf16 in registers and fed
// straight back as the A operand of Out^T = St^T A^T; the rows of the A tile
// are stored in LDS with the matching column permutation, so that both this
// product and the score product read them with 16-byte loads.
//
// LDS tiles per block
//   sA, sB   A and Bm row-major [row][feature'], feature' = feature with the two
//            middle quads of every 16 swapped (see above), row stride D+8
//   sBT,sCT  (w*Bm)^T and C^T, [feature][row], transposed in registers while
//            staging; 128-byte rows, XOR-swizzled so that both the 8-byte
//            transposing stores and the 16-byte operand loads are conflict free
//   sP       masked scores [q][key], row stride 72
//   sO       the Out tile, staged as bf16 in sB's storage (free once the scores
//            are done) with sB's layout, so every thread later overwrites, when
//            staging the next block, exactly the bytes it read itself: no
//            barrier is needed between the two.
//
// MFMA 32x32x16 bf16 register layout used throughout (lane l, i = l % 32,
// g = l / 32):  A operand: row i, k = 8g + e (e = 0..7);  B operand: column i,
// k = 8g + e;  C/D: column i, register v holds row 8*(v/4) + 4g + v%4.
#pragma once
#include "la_common.h"

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef uint32_t U4 __attribute__((ext_vector_type(4)));   // 16 bytes = 8 bf16
typedef uint32_t U2 __attribute__((ext_vector_type(2)));   //  8 bytes = 4 bf16

__device__ __forceinline__ uint32_t pack2_bf16(float lo, float hi)
{
    f32x2_t v = {lo, hi};
    bf16x2_t r = __builtin_convertvector(v, bf16x2_t);   // round-to-nearest-even
    return __builtin_bit_cast(uint32_t, r);
}
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
// (lo half of a, lo half of b) and (hi half of a, hi half of b) as one dword
__device__ __forceinline__ uint32_t pair_lo(uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x05040100u); }
__device__ __forceinline__ uint32_t pair_hi(uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x07060302u); }

__device__ __forceinline__ f32x16_t mfma32(const U4 &a, const U4 &b, f32x16_t c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                   __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}

// Scheduling fence between a batch of LDS operand loads and the MFMAs that use
// them: LDS instructions and MFMAs may not cross it, everything else may.
#define LA_BATCH_FENCE() __builtin_amdgcn_sched_barrier(0x476)

// Transposed-tile addressing, in bf16 elements: feature f (row), block row r.
//   physical row   = f with bits 0 and 3 swapped (so that the 16 features 8*sc+e
//                    written by one store instruction fall on both bank halves)
//   16-byte chunk  = (r / 8) ^ phi(f),  phi(f) = (f & 7) ^ ((f >> 4) & 7)
__device__ __forceinline__ int tt_row(int f) { return (f & ~9) | ((f & 1) << 3) | ((f >> 3) & 1); }
__device__ __forceinline__ int tt_phi(int f) { return (f & 7) ^ ((f >> 4) & 7); }

// Swish of the 8 bf16 values of a 16-byte chunk (fp32 inside, rounded back to bf16:
// the contractions see what they would see had the activated tensor been stored).
__device__ __forceinline__ U4 swish_u4(U4 r)
{
    U4 o;
#pragma unroll
    for (int j = 0; j < 4; ++j) o[j] = pack2_bf16(la_swish(bf16_lo(r[j])), la_swish(bf16_hi(r[j])));
    return o;
}
// 8 bf16 results times phi' of the 8 bf16 pre-activations in `x`
__device__ __forceinline__ U4 mul_swish_grad_u4(U4 r, U4 x)
{
    U4 o;
#pragma unroll
    for (int j = 0; j < 4; ++j)
        o[j] = pack2_bf16(bf16_lo(r[j]) * la_swish_grad(bf16_lo(x[j])),
                          bf16_hi(r[j]) * la_swish_grad(bf16_hi(x[j])));
    return o;
}

// sum of two chunks of 8 bf16 (fp32 add, one rounding)
__device__ __forceinline__ U4 add_u4(U4 r, U4 x)
{
    U4 o;
#pragma unroll
    for (int j = 0; j < 4; ++j)
        o[j] = pack2_bf16(bf16_lo(r[j]) + bf16_lo(x[j]), bf16_hi(r[j]) + bf16_hi(x[j]));
    return o;
}

template <int D>
struct Bf16Cfg {
    static constexpr int BK = 64;
    static constexpr int NW = D / 32;          // wavefronts per workgroup
    static constexpr int NT = NW * 64;
    static constexpr int LDN = D + 8;          // row stride of row-major tiles (elements)
    static constexpr int LDP = BK + 8;
    static constexpr int nA = BK * LDN, nB = BK * LDN, nBT = D * BK, nCT = D * BK, nP = BK * LDP;
    static constexpr size_t lds_bytes = 2 * (size_t)(nA + nB + nBT + nCT + nP);
};

// ACT: the launch may carry LA_ACT_* flags (Swish prologue / epilogue).
template <int D, bool REV, bool ACT>
__global__ __launch_bounds__(D * 2, 2) void la_scan_bf16(ScanLaunch launch, LaLambdas lams)
{
    using Cfg = Bf16Cfg<D>;
    constexpr int BK = Cfg::BK, NW = Cfg::NW;
    constexpr int LDN = Cfg::LDN, LDP = Cfg::LDP;
    constexpr int KS_D = D / 16;               // k-steps over the feature dim
    constexpr int KS_B = BK / 16;              // k-steps over the block rows (= 4)
    constexpr int MT_D = D / 32;               // 32-row tiles over the feature dim
    constexpr int CH = D / 8;                  // 16-byte chunks per row
    constexpr int NTILE = (3 + NW - 1) / NW;   // score tiles per wave (3 non-zero tiles)

    extern __shared__ __align__(16) uint16_t smem_bf16[];
    uint16_t *sA = smem_bf16;
    uint16_t *sB = sA + Cfg::nA;
    uint16_t *sBT = sB + Cfg::nB;
    uint16_t *sCT = sBT + Cfg::nBT;
    uint16_t *sP = sCT + Cfg::nCT;
    uint16_t *sO = sB;

    const int tid = threadIdx.x;
    const int w = tid >> 6, l = tid & 63, l32 = l & 31, g = l >> 5;
    const int sa = tid / CH, sc = tid % CH;    // staging: rows 4sa..4sa+3, chunk sc

    int item = blockIdx.x, role = 0;
    if (launch.nroles == 2) {
        const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
        role = slot & 1;
        item = (slot >> 1) * 8 + xcd;
        if (item >= launch.items) return;
    }
    const ScanArgs &a = launch.r[role];
    const int seg = item % a.S;
    const int scan = item / a.S;
    constexpr bool rev = REV;
    const float lg = lams.lg2[scan % a.H];
    auto pw = [lg](int k) -> float { return exp2f((float)k * lg); };

    const int seg_lo = seg * a.L;
    const int seg_hi = min(a.n, seg_lo + a.L);
    const int nblk = (seg_hi - seg_lo + BK - 1) / BK;

    const int act = ACT ? a.act : 0;
    // operand slabs: contiguous [scans, n, D] in the plain variants, free layouts otherwise
    const size_t base = (size_t)scan * a.n * D;
    const int bi = scan / a.H, hi = scan % a.H;
    auto slab = [&](const void *p, const LaLayout &l) -> uint16_t * {
        return (uint16_t *)p + (ACT ? (size_t)bi * l.bs + (size_t)hi * l.hs : base);
    };
    const uint16_t *gA = slab(a.A, a.lA);
    const uint16_t *gB = slab(a.Bm, a.lB);
    const uint16_t *gC = slab(a.C, a.lC);
    uint16_t *gO = slab(a.Out, a.lO);
    const int ldA = ACT ? a.lA.ld : D, ldB = ACT ? a.lB.ld : D, ldC = ACT ? a.lC.ld : D;
    const int ldO = ACT ? a.lO.ld : D;
    // tile fetched for the epilogue: the pre-activation (phi') or the previous Out (accumulate)
    const bool epi_e = ACT && (act & LA_ACT_OUT), epi_acc = ACT && (act & LA_ACT_ACC);
    const uint16_t *gE = epi_e ? slab(a.E, a.lE) : gO;
    const int ldE = epi_e ? a.lE.ld : ldO;
    // ---- per-lane constants --------------------------------------------------
    float wst[4];                              // state-update weight of staged rows
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int r = 4 * sa + i;
        wst[i] = rev ? pw(r) : pw(BK - 1 - r);
    }
    float lamBK = pw(BK);
    // (the activation variants have no entry point that hands a state back)
    const bool want_final = !REV && !ACT && a.st_out != nullptr && seg == a.S - 1;
    // row-major tiles: this thread's two 8-byte pieces of chunk sc
    const int nat_off = 16 * (sc >> 1) + 4 * (sc & 1);
    // transposed tiles, stores: feature f = 8sc + e lives in physical row
    // tt_row(f) = tw_row + ((e&1)<<3 | (e&6)) and chunk (sa>>1) ^ tt_phi(f) = tw_u ^ e
    const int tw_row = (((sc >> 1) << 4) | (sc & 1)) * BK + 4 * (sa & 1);
    int tw_u = 8 * ((sa >> 1) ^ ((sc >> 1) & 7));
    // transposed tiles, operand loads: feature f = 32m + l32 lives in physical row
    // 32m + tt_row(l32), and chunk (2ks+g) ^ tt_phi(f) = tr_pg ^ 2(ks ^ m)
    const int tr_row = tt_row(l32) * BK;
    int tr_pg = 8 * (((l32 & 7) ^ (l32 >> 4)) ^ g);

    float rsq[2];                              // inter-block scale of column q = 32mt + l32
    float mk[NTILE][16];                       // decay mask of this wave's score tiles
    {
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
            const int q = 32 * mt + l32;
            rsq[mt] = REV ? pw(BK - q) : pw(q + 1);
        }
#pragma unroll
        for (int ti = 0; ti < NTILE; ++ti) {
            int tile = w + ti * NW;            // 0,1,2 -> (kt,qt)
            int kt = REV ? (tile >= 1) : (tile == 2);
            int qt = REV ? (tile == 2) : (tile >= 1);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                int key = 32 * kt + 8 * (v >> 2) + 4 * g + (v & 3);
                int q = 32 * qt + l32;
                int dist = REV ? (key - q) : (q - key);
                mk[ti][v] = (dist >= 0) ? pw(dist) : 0.0f;
            }
        }
    }

    // ---- running state: St[i][j], j in this wave's slice ----------------------
    f32x16_t st[MT_D];
    // entering state: a segment state, or (first segment) the caller's carried state, or zero
    const float *gSt = la_entering_state(a, scan, seg, REV, lg, D * D);
    const bool has_init = gSt != nullptr;
    if (has_init && a.transpose_init) {
        // The stored state is that of the scan with Bm and C exchanged: copy it to LDS
        // with coalesced 16-byte loads (the tiles' storage is still unused) and read it
        // back transposed, so that this workgroup starts as quickly as its partner of
        // a paired launch and the two stay in step.
        float *sT = reinterpret_cast<float *>(smem_bf16);          // [D][D+1]
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
                int i = 32 * mt + 8 * (v >> 2) + 4 * g + (v & 3);
                st[mt][v] = sT[(32 * w + l32) * (D + 1) + i];
            }
        __syncthreads();
    } else {
#pragma unroll
        for (int mt = 0; mt < MT_D; ++mt)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                int i = 32 * mt + 8 * (v >> 2) + 4 * g + (v & 3);
                st[mt][v] = has_init ? gSt[(size_t)i * D + 32 * w + l32] : 0.0f;
            }
    }

    // ---- global -> register prefetch of one block -------------------------------
    // Rows past the segment end read the segment's last row instead (always in
    // bounds); they are zeroed when the block is staged, so that nothing here
    // consumes the loaded values and the loads stay in flight behind the compute.
    // Tiles that no other workgroup reads are loaded with the non-temporal hint (they
    // should not displace anything in L2): everything in a single-scan launch, the A
    // operand in a paired launch, whose Bm and C tiles the partner workgroup reads too.
    // (Measured: +3 % on the sweep; with the hint on the shared tiles as well, -6 %.)
    U4 ra[4], rb[4], rc[4];
    const bool nt_all = launch.nroles == 1;
    // (paired launch with the Swish epilogue: the dV scan's A operand is the tile whose
    // phi' the dK scan needs a little later)
    const bool nt_a = nt_all || !(ACT && role == 1);
    auto load_block = [&](int blk) {
        const int t0 = seg_lo + blk * BK;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int t = t0 + 4 * sa + i;
            const size_t row = (size_t)min(t, seg_hi - 1);
            const size_t off = row * D + 8 * sc;         // plain variants: one offset for all
            const U4 *pa = (const U4 *)(ACT ? gA + row * ldA + 8 * sc : gA + off);
            const U4 *pb = (const U4 *)(ACT ? gB + row * ldB + 8 * sc : gB + off);
            const U4 *pc = (const U4 *)(ACT ? gC + row * ldC + 8 * sc : gC + off);
            if (nt_all) {
                rb[i] = __builtin_nontemporal_load(pb);
                rc[i] = __builtin_nontemporal_load(pc);
            } else {
                rb[i] = *pb;
                rc[i] = *pc;
            }
            if (nt_a) ra[i] = __builtin_nontemporal_load(pa);
            else ra[i] = *pa;
        }
    };
    // ---- registers -> LDS, transposing C and the weighted Bm ---------------------
    auto stage_block = [&](int t0) {
        if (t0 + BK > seg_hi) {                 // partial block: zero padding (exact)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const bool ok = t0 + 4 * sa + i < seg_hi;
                const U4 z = {0u, 0u, 0u, 0u};
                rb[i] = ok ? rb[i] : z;
                rc[i] = ok ? rc[i] : z;
                ra[i] = ok ? ra[i] : z;
            }
        }
        if (ACT) {                              // phi(0) = 0: the zero padding stays zero
            if (act & LA_ACT_A) {
#pragma unroll
                for (int i = 0; i < 4; ++i) ra[i] = swish_u4(ra[i]);
            }
            if (act & LA_ACT_BM) {
#pragma unroll
                for (int i = 0; i < 4; ++i) rb[i] = swish_u4(rb[i]);
            }
            if (act & LA_ACT_C) {
#pragma unroll
                for (int i = 0; i < 4; ++i) rc[i] = swish_u4(rc[i]);
            }
        }
        {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                uint16_t *pa = sA + (4 * sa + i) * LDN + nat_off;
                uint16_t *pb = sB + (4 * sa + i) * LDN + nat_off;
                *(U2 *)(pa) = U2{ra[i][0], ra[i][1]};
                *(U2 *)(pa + 8) = U2{ra[i][2], ra[i][3]};
                *(U2 *)(pb) = U2{rb[i][0], rb[i][1]};
                *(U2 *)(pb + 8) = U2{rb[i][2], rb[i][3]};
            }
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            // element e of each of the 4 rows -> 4 consecutive block rows of feature 8sc+e
            const int j = e >> 1;
            float b0, b1, b2, b3;
            U2 tb, tc;
            if (e & 1) {
                b0 = bf16_hi(rb[0][j]); b1 = bf16_hi(rb[1][j]);
                b2 = bf16_hi(rb[2][j]); b3 = bf16_hi(rb[3][j]);
                tc[0] = pair_hi(rc[0][j], rc[1][j]);
                tc[1] = pair_hi(rc[2][j], rc[3][j]);
            } else {
                b0 = bf16_lo(rb[0][j]); b1 = bf16_lo(rb[1][j]);
                b2 = bf16_lo(rb[2][j]); b3 = bf16_lo(rb[3][j]);
                tc[0] = pair_lo(rc[0][j], rc[1][j]);
                tc[1] = pair_lo(rc[2][j], rc[3][j]);
            }
            tb[0] = pack2_bf16(b0 * wst[0], b1 * wst[1]);
            tb[1] = pack2_bf16(b2 * wst[2], b3 * wst[3]);
            const int off = tw_row + (((e & 1) << 3) | (e & 6)) * BK + (tw_u ^ (8 * e));
            *(U2 *)(sBT + off) = tb;
            *(U2 *)(sCT + off) = tc;
        }
    };

    load_block(rev ? nblk - 1 : 0);

    for (int ib = 0; ib < nblk; ++ib) {
        const int blk = rev ? (nblk - 1 - ib) : ib;
        const int t0 = seg_lo + blk * BK;
        // the swizzle terms are re-derived per block (one XOR each) instead of living
        // in a register per address for the whole loop
        asm volatile("" : "+v"(tw_u), "+v"(tr_pg));
        if (want_final && t0 + BK > seg_hi) {
            // The state handed back must be the one after the last real token: in the
            // final, partial block of m rows weight row r by lambda^(m-1-r) and decay the
            // old state by lambda^m instead of padding the block out to BK rows.
            const int m = seg_hi - t0;
#pragma unroll
            for (int i = 0; i < 4; ++i) wst[i] = pw(max(m - 1 - (4 * sa + i), 0));
            lamBK = pw(m);
        }
        stage_block(t0);
        // the registers are free again: prefetch before waiting for the other waves
        if (ib + 1 < nblk) load_block(rev ? blk - 1 : blk + 1);
        __syncthreads();

        U4 cf[KS_B];                            // C^T fragments of this wave's slice
        auto load_cf = [&]() {
#pragma unroll
            for (int ks = 0; ks < KS_B; ++ks)
                cf[ks] = *(const U4 *)(sCT + 32 * w * BK + tr_row + (tr_pg ^ (16 * (ks ^ (w & 3)))));
        };

        // Operand fragments are read from LDS in batches of eight 16-byte loads that
        // are all issued before the MFMAs that consume them (a scheduling barrier keeps
        // the compiler from sinking each load next to its use): the LDS latency is paid
        // once per batch instead of once per MFMA.
        f32x16_t acc[2];
        {
            // ---- scores: S^T tile (kt, qt) = Bm[kt] A[qt]^T, masked, to LDS as P[q][key]
#pragma unroll
            for (int ti = 0; ti < NTILE; ++ti) {
                const int tile = w + ti * NW;
                if (tile < 3) {
                    const int kt = REV ? (tile >= 1) : (tile == 2);
                    const int qt = REV ? (tile == 2) : (tile >= 1);
                    const uint16_t *pa = sB + (32 * kt + l32) * LDN + 8 * g;
                    const uint16_t *pb = sA + (32 * qt + l32) * LDN + 8 * g;
                    f32x16_t s = {0};
#pragma unroll
                    for (int h = 0; h < KS_D / 4; ++h) {
                        U4 fa[4], fb[4];
#pragma unroll
                        for (int k = 0; k < 4; ++k) {
                            fa[k] = *(const U4 *)(pa + 16 * (4 * h + k));
                            fb[k] = *(const U4 *)(pb + 16 * (4 * h + k));
                        }
                        LA_BATCH_FENCE();
#pragma unroll
                        for (int k = 0; k < 4; ++k) s = mfma32(fa[k], fb[k], s);
                    }
#pragma unroll
                    for (int v4 = 0; v4 < 4; ++v4) {
                        U2 p;
                        p[0] = pack2_bf16(s[4 * v4 + 0] * mk[ti][4 * v4 + 0],
                                          s[4 * v4 + 1] * mk[ti][4 * v4 + 1]);
                        p[1] = pack2_bf16(s[4 * v4 + 2] * mk[ti][4 * v4 + 2],
                                          s[4 * v4 + 3] * mk[ti][4 * v4 + 3]);
                        *(U2 *)(sP + (32 * qt + l32) * LDP + 32 * kt + 8 * v4 + 4 * g) = p;
                    }
                }
            }
            // ---- inter block: acc^T = (St^T A^T) * scale(q).  The state operand is made
            // from the accumulator registers k-step by k-step and used for both q tiles.
            {
                f32x16_t x0 = {0}, x1 = {0};
                const uint16_t *p0 = sA + l32 * LDN + 8 * g;
                const uint16_t *p1 = sA + (32 + l32) * LDN + 8 * g;
#pragma unroll
                for (int h = 0; h < KS_D / 2; ++h) {
                    U4 f0[2], f1[2];
#pragma unroll
                    for (int k = 0; k < 2; ++k) {
                        f0[k] = *(const U4 *)(p0 + 16 * (2 * h + k));
                        f1[k] = *(const U4 *)(p1 + 16 * (2 * h + k));
                    }
                    LA_BATCH_FENCE();
#pragma unroll
                    for (int k = 0; k < 2; ++k) {
                        const int ks = 2 * h + k, mt = ks >> 1, h8 = 8 * (ks & 1);
                        U4 so;
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            so[e] = pack2_bf16(st[mt][h8 + 2 * e], st[mt][h8 + 2 * e + 1]);
                        x0 = mfma32(so, f0[k], x0);
                        x1 = mfma32(so, f1[k], x1);
                    }
                }
#pragma unroll
                for (int v = 0; v < 16; ++v) { x0[v] *= rsq[0]; x1[v] *= rsq[1]; }
                acc[0] = x0;
                acc[1] = x1;
            }
            __syncthreads();                    // P is complete; sB is free from here on
            // ---- intra block: acc^T += C^T P^T
            {
                U4 fp[2][KS_B];
                load_cf();
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                    for (int ks = 0; ks < KS_B; ++ks) {
                        const int ktile = ks >> 1;
                        const bool live = REV ? (ktile >= mt) : (ktile <= mt);
                        if (live) fp[mt][ks] = *(const U4 *)(sP + (32 * mt + l32) * LDP + 16 * ks + 8 * g);
                    }
                LA_BATCH_FENCE();
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                    for (int ks = 0; ks < KS_B; ++ks) {
                        const int ktile = ks >> 1;
                        const bool live = REV ? (ktile >= mt) : (ktile <= mt);
                        if (live) acc[mt] = mfma32(cf[ks], fp[mt][ks], acc[mt]);
                    }
            }
            // ---- Out tile -> sO (bf16, sB's layout): lane holds 4 consecutive features per v4
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int v4 = 0; v4 < 4; ++v4) {
                    U2 o;
                    o[0] = pack2_bf16(acc[mt][4 * v4 + 0], acc[mt][4 * v4 + 1]);
                    o[1] = pack2_bf16(acc[mt][4 * v4 + 2], acc[mt][4 * v4 + 3]);
                    const int quad = 2 * (v4 & 1) + g;                 // quad of the 16-group
                    const int pquad = (quad == 1) ? 2 : (quad == 2 ? 1 : quad);
                    *(U2 *)(sO + (32 * mt + l32) * LDN + 32 * w + 16 * (v4 >> 1) + 4 * pquad) = o;
                }
        }

        // Epilogue operand: the pre-activation tile whose phi' scales Out.  Loaded here, where
        // the Out accumulators have just died, and used after the state update.
        U4 re[4];
        if (epi_e || epi_acc) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
            {
                const U4 *pe = (const U4 *)(gE + (size_t)min(t0 + 4 * sa + i, seg_hi - 1) * ldE + 8 * sc);
                re[i] = nt_all ? __builtin_nontemporal_load(pe) : *pe;
            }
        }
        // ---- state update: St = lambda^BK St + (w Bm)^T C ---------------------------
#pragma unroll
        for (int mt = 0; mt < MT_D; ++mt) {
            U4 fa[KS_B];
#pragma unroll
            for (int ks = 0; ks < KS_B; ++ks)
                fa[ks] = *(const U4 *)(sBT + 32 * mt * BK + tr_row + (tr_pg ^ (16 * (ks ^ mt))));
            LA_BATCH_FENCE();
            f32x16_t s = st[mt];
#pragma unroll
            for (int v = 0; v < 16; ++v) s[v] *= lamBK;
#pragma unroll
            for (int ks = 0; ks < KS_B; ++ks) s = mfma32(fa[ks], cf[ks], s);
            st[mt] = s;
        }

        {
            __syncthreads();                    // sO complete; every LDS tile of this block is dead
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int t = t0 + 4 * sa + i;
                const uint16_t *po = sO + (4 * sa + i) * LDN + nat_off;
                U2 lo = *(const U2 *)(po);
                U2 hi = *(const U2 *)(po + 8);
                U4 out = {lo[0], lo[1], hi[0], hi[1]};
                if (epi_e) out = mul_swish_grad_u4(out, re[i]);
                else if (epi_acc) out = add_u4(out, re[i]);
                if (t < seg_hi) __builtin_nontemporal_store(out, (U4 *)(gO + (size_t)t * ldO + 8 * sc));
            }
        }
    }

    if (want_final) {
        float *dst = a.st_out + (size_t)scan * (D * D);
#pragma unroll
        for (int mt = 0; mt < MT_D; ++mt)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                int i = 32 * mt + 8 * (v >> 2) + 4 * g + (v & 3);
                dst[(size_t)i * D + 32 * w + l32] = st[mt][v];
            }
    }
}
