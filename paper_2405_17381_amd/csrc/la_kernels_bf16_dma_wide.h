// Forward block scan with a query / key feature twice as wide as the value feature
// (d_k = 256, d_v = 128: LRPE-d's cos / sin features, Sec. 4.1), on the direct-to-LDS machinery
// of la_kernels_bf16_dma.h.  One kernel holds the whole non-square 256 x 128 state, so that
//     O[t] = sum_{s <= t} lambda^(t-s) (Qw[t] . Kw[s]) V[s]
// costs one pass over Qw, Kw, V and one write of O (6 tensor passes of d_v-wide rows) instead of
// two accumulated scans over the cos and the sin half (9 passes, O rounded to bf16 in between).
//
// Same structure as la_scan_bf16_dma: 32-row blocks, three LDS stages filled by global -> LDS
// loads (A and Bm tiles 32 x 256 = 16 KB each, C tile 32 x 128 = 8 KB), row reads for the
// contractions over the 256 features, transposing reads for those over the tokens, wave w owns
// value features [32w, 32w + 32) of Out and of the state (eight 32 x 32 accumulator tiles), the
// state feeds the inter product from registers after a lane swap, the masked scores stay in
// registers.  One workgroup per compute unit (128 KB of LDS, up to 512 registers per lane).
// Whole sequences only (one segment, zero entering state): the launch code falls back to the
// accumulated scans whenever the planner cuts the sequence.
#pragma once
#include "la_kernels_bf16_dma.h"

struct DmaWideCfg {
    static constexpr int DK = 256, DV = 128, BK = 32, NS = 3, NW = 4, NT = 256;
    static constexpr int TILE_K_BYTES = BK * DK * 2;         // A, Bm: 16384
    static constexpr int TILE_V_BYTES = BK * DV * 2;         // C: 8192
    static constexpr int STAGE_BYTES = 2 * TILE_K_BYTES + TILE_V_BYTES;
    static constexpr int SO_BYTES = BK * DV * 2;
    static constexpr size_t lds_bytes = (size_t)NS * STAGE_BYTES + SO_BYTES;   // 131072
};

__global__ __launch_bounds__(256, 1) void la_scan_bf16_dma_wide(ScanLaunch launch, LaLambdas lams)
{
    using Cfg = DmaWideCfg;
    constexpr int DK = Cfg::DK, DV = Cfg::DV, BK = Cfg::BK, NS = Cfg::NS, PF = NS - 1;
    constexpr int KS_B = BK / 16;              // k-steps over the block rows (2)
    constexpr int MT_D = DK / 32;              // 32-row tiles of the state (8)
    constexpr int LOADS = 4 + 4 + 2;           // direct loads per wave and block (A, Bm, C)
    constexpr int ST = 2;                      // store instructions per wave and block

    extern __shared__ __align__(16) unsigned char smem_dma[];

    const int tid = threadIdx.x;
    const int l = tid & 63, l32 = l & 31, g = l >> 5;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);

    const ScanArgs &a = launch.r[0];
    const int scan = blockIdx.x;               // one segment per scan
    const float lg = lams.lg2[scan % a.H];
    auto pw = [lg](int k) -> float { return exp2f((float)k * lg); };
    const int seg_hi = a.n;
    const int nblk = (a.n + BK - 1) / BK;

    const uint16_t *gA = (const uint16_t *)a.A + (size_t)scan * a.n * DK;
    const uint16_t *gB = (const uint16_t *)a.Bm + (size_t)scan * a.n * DK;
    const uint16_t *gC = (const uint16_t *)a.C + (size_t)scan * a.n * DV;
    uint16_t *gO = (uint16_t *)a.Out + (size_t)scan * a.n * DV;

    float mk[16], wt[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int key = 8 * (v >> 2) + 4 * g + (v & 3);
        const int dist = l32 - key;
        mk[v] = dist >= 0 ? pw(dist) : 0.0f;
        wt[v] = pw(BK - 1 - key);
    }
    const float rsq = pw(l32 + 1);
    const float lamBK = pw(BK);

    // row reads of the 512-byte rows of A and Bm: row l32, chunk 2 ks + g (0..31); the swizzle
    // touches the low four bits of the chunk index only
    const int rk_base = l32 * 512;
    const int ro_sw = dma_sw(l32) ^ g;
    const int a4 = l & 3, b4 = (l >> 2) & 3, h16 = (l >> 4) & 1;
    const int trk_base = (4 * g + b4) * 512 + 8 * (a4 & 1);      // transposing reads of Bm (512-byte rows)
    const int trv_base = (4 * g + b4) * 256 + 8 * (a4 & 1);      // ... of C (256-byte rows)
    const int tr_sw = (2 * h16 + (a4 >> 1)) ^ (4 * b4 + g);
    // direct loads.  A, Bm: load slot ii = 4w + j covers tile rows 2 ii, 2 ii + 1 (lane -> row
    // l >> 5, chunk l & 31); C: slot ii = 2w + j covers rows 4 ii .. 4 ii + 3 as in the square kernel.
    int krow[4], kcol[4], vrow[2], vcol[2];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        krow[j] = 2 * (4 * w + j) + (l >> 5);
        kcol[j] = 8 * ((l & 31) ^ dma_sw(krow[j]));
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        vrow[j] = 4 * (2 * w + j) + (l >> 4);
        vcol[j] = 8 * ((l & 15) ^ dma_sw(vrow[j]));
    }
    unsigned char *sO = smem_dma + NS * Cfg::STAGE_BYTES;
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(la_lds_void *)smem_dma);

    f32x16_t st[MT_D];
#pragma unroll
    for (int mt = 0; mt < MT_D; ++mt)
#pragma unroll
        for (int v = 0; v < 16; ++v) st[mt][v] = 0.0f;

    auto issue = [&](int ib, int stage) {
        const int t0 = ib * BK;
        const uint32_t sb = lds0 + stage * Cfg::STAGE_BYTES;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const size_t off = (size_t)min(t0 + krow[j], seg_hi - 1) * DK + kcol[j];
            const uint32_t dst = sb + (4 * w + j) * 1024;
            dma_load16<true>(gA + off, dst);
            dma_load16<true>(gB + off, dst + Cfg::TILE_K_BYTES);
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const size_t off = (size_t)min(t0 + vrow[j], seg_hi - 1) * DV + vcol[j];
            dma_load16<true>(gC + off, sb + 2 * Cfg::TILE_K_BYTES + (2 * w + j) * 1024);
        }
    };
    auto store_out = [&](int t0) {
        const int last = min(BK, seg_hi - t0) - 1;
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            const int row = min(8 * w + 4 * p + (l >> 4), last), ch = l & 15;
            const U4 o = *(const U4 *)(sO + row * 256 + ((ch ^ (row & 15)) << 4));
            __builtin_nontemporal_store(o, (U4 *)(gO + (size_t)(t0 + row) * DV + 8 * ch));
        }
    };

#pragma unroll
    for (int i = 0; i < PF; ++i)
        if (i < nblk) issue(i, i);

    int stage = 0;
    for (int ib = 0; ib < nblk; ++ib) {
        const int t0 = ib * BK;
        unsigned char *sb = smem_dma + stage * Cfg::STAGE_BYTES;
        if (nblk < 2 * PF + 1 || ib + 1 >= nblk) {
            la_wait_vm<0>();
        } else {
            const int young = min(PF - 1, nblk - 1 - ib);
            const int olds = min(PF - 1, ib);
            la_wait_vm_le<(PF - 1) * (LOADS + ST)>(LOADS * young + ST * olds);
        }
        if (t0 + BK > seg_hi) {                 // partial block: zero padding (exact)
            const U4 z = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (t0 + krow[j] >= seg_hi) {
                    unsigned char *dst = sb + (4 * w + j) * 1024 + 16 * l;
                    *(U4 *)dst = z;
                    *(U4 *)(dst + Cfg::TILE_K_BYTES) = z;
                }
#pragma unroll
            for (int j = 0; j < 2; ++j)
                if (t0 + vrow[j] >= seg_hi)
                    *(U4 *)(sb + 2 * Cfg::TILE_K_BYTES + (2 * w + j) * 1024 + 16 * l) = z;
        }
        LA_LDS_BARRIER();
        if (ib + PF < nblk) issue(ib + PF, stage >= 1 ? stage - 1 : NS - 1);

        const unsigned char *sA = sb, *sB = sb + Cfg::TILE_K_BYTES, *sC = sb + 2 * Cfg::TILE_K_BYTES;

        // scores and inter product over the 256 features, a quarter of the k range at a time
        f32x16_t s = {0}, x = {0};
#pragma unroll
        for (int h = 0; h < 4; ++h) {
            U4 fa[4], fb[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                fa[k] = *(const U4 *)(sA + rk_base + (((2 * (4 * h + k)) ^ ro_sw) << 4));
                fb[k] = *(const U4 *)(sB + rk_base + (((2 * (4 * h + k)) ^ ro_sw) << 4));
            }
            LA_BATCH_FENCE();
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int ks = 4 * h + k, mt = ks >> 1, h8 = 8 * (ks & 1);
                s = mfma32(fb[k], fa[k], s);
                const uint32_t x0 = pack2_bf16(st[mt][h8 + 0], st[mt][h8 + 1]);
                const uint32_t x1 = pack2_bf16(st[mt][h8 + 2], st[mt][h8 + 3]);
                const uint32_t y0 = pack2_bf16(st[mt][h8 + 4], st[mt][h8 + 5]);
                const uint32_t y1 = pack2_bf16(st[mt][h8 + 6], st[mt][h8 + 7]);
                const auto s0 = __builtin_amdgcn_permlane32_swap(x0, y0, false, false);
                const auto s1 = __builtin_amdgcn_permlane32_swap(x1, y1, false, false);
                const U4 so = {s0[0], s1[0], s0[1], s1[1]};
                x = mfma32(so, fa[k], x);
            }
        }
        U4 cf[KS_B], cw[KS_B], pk[KS_B];
#pragma unroll
        for (int ks = 0; ks < KS_B; ++ks) {
            const unsigned char *p = sC + trv_base + 16 * ks * 256;
            const U2 lo = lds_read_tr(p + ((((4 * w) ^ tr_sw)) << 4));
            const U2 hi = lds_read_tr(p + 8 * 256 + ((((4 * w) ^ tr_sw ^ 2)) << 4));
            cf[ks] = U4{lo[0], lo[1], hi[0], hi[1]};
        }
#pragma unroll
        for (int ks = 0; ks < KS_B; ++ks)
#pragma unroll
            for (int e = 0; e < 4; ++e)
                pk[ks][e] = pack2_bf16(s[8 * ks + 2 * e] * mk[8 * ks + 2 * e],
                                       s[8 * ks + 2 * e + 1] * mk[8 * ks + 2 * e + 1]);
#pragma unroll
        for (int v = 0; v < 16; ++v) x[v] *= rsq;
#pragma unroll
        for (int ks = 0; ks < KS_B; ++ks) x = mfma32(cf[ks], pk[ks], x);
#pragma unroll
        for (int v4 = 0; v4 < 4; ++v4) {
            U2 o;
            o[0] = pack2_bf16(x[4 * v4 + 0], x[4 * v4 + 1]);
            o[1] = pack2_bf16(x[4 * v4 + 2], x[4 * v4 + 3]);
            *(U2 *)(sO + l32 * 256 + (((4 * w + v4) ^ (l32 & 15)) << 4) + 8 * g) = o;
        }
#pragma unroll
        for (int ks = 0; ks < KS_B; ++ks)
#pragma unroll
            for (int e = 0; e < 4; ++e)
                cw[ks][e] = pack2_bf16(bf16_lo(cf[ks][e]) * wt[8 * ks + 2 * e],
                                       bf16_hi(cf[ks][e]) * wt[8 * ks + 2 * e + 1]);
        // state update: St = lambda^BK St + Bm^T (w C), eight row tiles
#pragma unroll
        for (int mt = 0; mt < MT_D; ++mt) {
            U4 bt[KS_B];
#pragma unroll
            for (int ks = 0; ks < KS_B; ++ks) {
                const unsigned char *p = sB + trk_base + 16 * ks * 512;
                const U2 lo = lds_read_tr(p + ((((4 * mt) ^ tr_sw)) << 4));
                const U2 hi = lds_read_tr(p + 8 * 512 + ((((4 * mt) ^ tr_sw ^ 2)) << 4));
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
        LA_LDS_BARRIER();
        store_out(t0);
        stage = stage + 1 < NS ? stage + 1 : 0;
    }
}
