// bf16 segment-state pre-pass: the local end state of every segment,
//     forward scans   S = sum_r lambda^(b-1-r)  Bm[r] C[r]^T   (r in [a, b), b = a + L)
//     reverse scans   S = sum_r lambda^(r-a)    Bm[r] C[r]^T
// (App. C's KV_t / dKV_t at segment granularity, before the segment scan chains
// them).  It is the state-update contraction of the block scan alone, so the
// per-block work is one dependent chain: stage a 64-row block of Bm and C
// transposed into LDS, then D/32 x 4 MFMAs per wave.  To keep that chain short:
//   * the decay is folded into the staging weights (row r of block k is weighted
//     by its full distance to the segment's end), so the state is never rescaled;
//   * the transposed tiles are double buffered in LDS: one barrier per block;
//   * blocks whose weights are below 2^-skip_bits are not read at all.
// One launch can hold two independent pre-passes (roles), one after the other in
// the grid, each with its own direction; heads are dispatched by decreasing lambda
// so that the long chains start first.
#pragma once
#include <type_traits>

#include "la_kernels_bf16.h"

template <int D>
struct PrepassCfg {
    static constexpr int BK = 64;
    static constexpr int NT = D * 2;
    static constexpr int nT = D * BK;                       // one transposed tile (elements)
    static constexpr size_t lds_bytes = 2 * (size_t)(4 * nT);   // 2 buffers x (Bm^T, C^T)
};

template <int D, bool ACT>
__global__ __launch_bounds__(D * 2, 2) void la_prepass_bf16(ScanLaunch launch, LaLambdas lams)
{
    using Cfg = PrepassCfg<D>;
    constexpr int BK = Cfg::BK;
    constexpr int KS_B = BK / 16, MT_D = D / 32, CH = D / 8;

    extern __shared__ __align__(16) uint16_t smem_pre[];

    const int tid = threadIdx.x;
    const int w = tid >> 6, l = tid & 63, l32 = l & 31, g = l >> 5;
    const int sa = tid / CH, sc = tid % CH;

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

    const size_t base = (size_t)scan * a.n * D;
    const int bi = scan / a.H, hi = scan % a.H;
    const uint16_t *gB = (const uint16_t *)a.Bm + (ACT ? (size_t)bi * a.lB.bs + (size_t)hi * a.lB.hs : base);
    const uint16_t *gC = (const uint16_t *)a.C + (ACT ? (size_t)bi * a.lC.bs + (size_t)hi * a.lC.hs : base);
    const int ldB = ACT ? a.lB.ld : D, ldC = ACT ? a.lC.ld : D;
    float *gSt = a.states + ((size_t)scan * a.S + seg) * (size_t)(D * D);

    float wrow[4];                                           // weight of staged rows inside a block
#pragma unroll
    for (int i = 0; i < 4; ++i) wrow[i] = rev ? pw(4 * sa + i) : pw(BK - 1 - (4 * sa + i));
    const int tw_row = (((sc >> 1) << 4) | (sc & 1)) * BK + 4 * (sa & 1);
    int tw_u = 8 * ((sa >> 1) ^ ((sc >> 1) & 7));
    const int tr_row = tt_row(l32) * BK;
    int tr_pg = 8 * (((l32 & 7) ^ (l32 >> 4)) ^ g);

    f32x16_t st[MT_D];
#pragma unroll
    for (int mt = 0; mt < MT_D; ++mt)
#pragma unroll
        for (int v = 0; v < 16; ++v) st[mt][v] = 0.0f;

    // NSLOT blocks are kept in flight (registers): the per-block compute is shorter
    // than the HBM latency, so one block ahead would leave the chain latency-bound.
    constexpr int NSLOT = 4;
    U4 rb_all[NSLOT][4], rc_all[NSLOT][4];
    const auto blk_of = [&](int ib) { return rev ? (nblk - 1 - ib) : ib; };
    auto load_block = [&](auto slot_c, int ib) {
        constexpr int slot = decltype(slot_c)::value;
        const int t0 = seg_lo + blk_of(ib) * BK;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const size_t row = (size_t)min(t0 + 4 * sa + i, seg_hi - 1);
            const size_t off = row * D + 8 * sc;             // plain variant: one offset for both
            rb_all[slot][i] = __builtin_nontemporal_load((const U4 *)(ACT ? gB + row * ldB + 8 * sc : gB + off));
            rc_all[slot][i] = __builtin_nontemporal_load((const U4 *)(ACT ? gC + row * ldC + 8 * sc : gC + off));
        }
    };

    auto iterate = [&](auto slot_c, int ib) {
        constexpr int slot = decltype(slot_c)::value;
        U4 (&rb)[4] = rb_all[slot];
        U4 (&rc)[4] = rc_all[slot];
        const int blk = blk_of(ib);
        const int t0 = seg_lo + blk * BK;
        asm volatile("" : "+v"(tw_u), "+v"(tr_pg));
        uint16_t *sBT = smem_pre + (ib & 1) * (2 * Cfg::nT);
        uint16_t *sCT = sBT + Cfg::nT;
        // distance of this block to the segment's far end, folded into the row weights
        const float mu = rev ? pw(blk * BK) : pw((nblk - 1 - blk) * BK);
        if (t0 + BK > seg_hi) {                              // partial block: zero padding (exact)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const bool ok = t0 + 4 * sa + i < seg_hi;
                const U4 z = {0u, 0u, 0u, 0u};
                rb[i] = ok ? rb[i] : z;
                rc[i] = ok ? rc[i] : z;
            }
        }
        if (ACT) {                                           // Swish prologue, as the block scan's
            if (a.act & LA_ACT_BM) {
#pragma unroll
                for (int i = 0; i < 4; ++i) rb[i] = swish_u4(rb[i]);
            }
            if (a.act & LA_ACT_C) {
#pragma unroll
                for (int i = 0; i < 4; ++i) rc[i] = swish_u4(rc[i]);
            }
        }
        const float w0 = wrow[0] * mu, w1 = wrow[1] * mu, w2 = wrow[2] * mu, w3 = wrow[3] * mu;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
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
            tb[0] = pack2_bf16(b0 * w0, b1 * w1);
            tb[1] = pack2_bf16(b2 * w2, b3 * w3);
            const int off = tw_row + (((e & 1) << 3) | (e & 6)) * BK + (tw_u ^ (8 * e));
            *(U2 *)(sBT + off) = tb;
            *(U2 *)(sCT + off) = tc;
        }
        // One barrier per block: the other buffer was last read in the previous
        // iteration, which every wave finished before it arrived here.
        __syncthreads();
        if (ib + NSLOT < nblk) load_block(slot_c, ib + NSLOT);

        U4 cf[KS_B];
#pragma unroll
        for (int ks = 0; ks < KS_B; ++ks)
            cf[ks] = *(const U4 *)(sCT + 32 * w * BK + tr_row + (tr_pg ^ (16 * (ks ^ (w & 3)))));
#pragma unroll
        for (int mt = 0; mt < MT_D; ++mt) {
            U4 fa[KS_B];
#pragma unroll
            for (int ks = 0; ks < KS_B; ++ks)
                fa[ks] = *(const U4 *)(sBT + 32 * mt * BK + tr_row + (tr_pg ^ (16 * (ks ^ mt))));
            LA_BATCH_FENCE();
#pragma unroll
            for (int ks = 0; ks < KS_B; ++ks) st[mt] = mfma32(fa[ks], cf[ks], st[mt]);
        }
    };

    using S0 = std::integral_constant<int, 0>;
    using S1 = std::integral_constant<int, 1>;
    using S2 = std::integral_constant<int, 2>;
    using S3 = std::integral_constant<int, 3>;
    load_block(S0{}, ib0);
    if (ib0 + 1 < nblk) load_block(S1{}, ib0 + 1);
    if (ib0 + 2 < nblk) load_block(S2{}, ib0 + 2);
    if (ib0 + 3 < nblk) load_block(S3{}, ib0 + 3);
    for (int ib = ib0; ib < nblk; ib += NSLOT) {
        iterate(S0{}, ib);
        if (ib + 1 < nblk) iterate(S1{}, ib + 1);
        if (ib + 2 < nblk) iterate(S2{}, ib + 2);
        if (ib + 3 < nblk) iterate(S3{}, ib + 3);
    }

#pragma unroll
    for (int mt = 0; mt < MT_D; ++mt)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int i = 32 * mt + 8 * (v >> 2) + 4 * g + (v & 3);
            gSt[(size_t)i * D + 32 * w + l32] = st[mt][v];
        }
}
