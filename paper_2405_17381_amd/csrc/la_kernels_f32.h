// fp32 path: the block loop of Alg. 5 / Alg. 6 taken literally, all-fp32 FMA
// arithmetic, one workgroup of 256 threads per (scan, segment).  Tiles of A,
// Bm, C, the masked score tile and the running state all live in LDS.
// This kernel exists for fp32 parity (tolerance 1e-4), not for speed: it serves d = 64
// (64-row blocks) and, when LA_F32_PLAIN is set, d = 128 as a second implementation to
// compare the matrix-core fp32 kernel (la_kernels_f32m.h) against.
#pragma once
#include "la_common.h"

template <int D, int BK>
struct F32Cfg {
    static constexpr int NT = 256;
    static constexpr int LD = D + 1;            // padded row stride (floats)
    static constexpr int LS = BK + 1;
    static constexpr int RI = BK / 16;          // block rows per thread
    static constexpr int CJ = D / 16;           // feature columns per thread
    static constexpr size_t lds_bytes =
        sizeof(float) * (size_t)(3 * BK * LD + BK * LS + D * LD + (BK + 1));
};

template <int D, int BK, bool REV, bool STATE_ONLY>
__global__ __launch_bounds__(256) void la_scan_f32(ScanLaunch launch, LaLambdas lams)
{
    // two roles (two independent pre-passes in one launch) follow one another in the grid
    const int role = launch.nroles == 2 ? (int)(blockIdx.x / launch.items) : 0;
    const int item = launch.nroles == 2 ? (int)(blockIdx.x % launch.items) : (int)blockIdx.x;
    const ScanArgs &a = launch.r[role];
    using Cfg = F32Cfg<D, BK>;
    constexpr int LD = Cfg::LD, LS = Cfg::LS, RI = Cfg::RI, CJ = Cfg::CJ;
    extern __shared__ float smem_f32[];
    float *sA = smem_f32;
    float *sB = sA + BK * LD;
    float *sC = sB + BK * LD;
    float *sS = sC + BK * LD;
    float *sKV = sS + BK * LS;
    float *sPw = sKV + D * LD;

    const int tid = threadIdx.x;
    const int ty = tid >> 4, tx = tid & 15;
    const int seg = item % a.S;
    int scan = item / a.S;
    if (STATE_ONLY) {
        const int b = scan % a.B, hi = scan / a.B;
        scan = b * a.H + lams.order[hi];
    }
    const float lam = lams.v[scan % a.H];

    const int seg_lo = seg * a.L;
    const int seg_hi = min(a.n, seg_lo + a.L);
    const bool rev = STATE_ONLY ? (a.rev != 0) : REV;
    if (STATE_ONLY) {
        // the state leaving the last (forward) / first (reverse) segment is never used
        if (!rev && seg == a.S - 1) return;
        if (rev && seg == 0) return;
    }
    const int nblk = (seg_hi - seg_lo + BK - 1) / BK;

    // operand slabs (layouts are filled in for every launch; contiguous by default)
    const int bi = scan / a.H, hi = scan % a.H;
    const float *gA = (const float *)a.A + (size_t)bi * a.lA.bs + (size_t)hi * a.lA.hs;
    const float *gB = (const float *)a.Bm + (size_t)bi * a.lB.bs + (size_t)hi * a.lB.hs;
    const float *gC = (const float *)a.C + (size_t)bi * a.lC.bs + (size_t)hi * a.lC.hs;
    float *gO = (float *)a.Out + (size_t)bi * a.lO.bs + (size_t)hi * a.lO.hs;
    const float *gE = (a.act & LA_ACT_OUT) ? (const float *)a.E + (size_t)bi * a.lE.bs + (size_t)hi * a.lE.hs : gA;
    const int ldA = a.lA.ld, ldB = a.lB.ld, ldC = a.lC.ld, ldO = a.lO.ld, ldE = a.lE.ld;
    float *gSt = a.states ? a.states + ((size_t)scan * a.S + seg) * (size_t)(D * D) : nullptr;

    // lambda^k, k = 0..BK, evaluated in double then rounded once
    for (int k = tid; k <= BK; k += 256) sPw[k] = (float)pow((double)lam, (double)k);
    // initial state
    const float *gIn = STATE_ONLY ? nullptr : la_entering_state(a, scan, seg, REV, lams.lg2[scan % a.H], D * D);
    const bool has_init = gIn != nullptr;
    const bool want_final = !STATE_ONLY && !REV && a.st_out != nullptr && seg == a.S - 1;
    for (int e = tid; e < D * D; e += 256) {
        int i = e / D, j = e % D;
        sKV[i * LD + j] = has_init ? (a.transpose_init ? gIn[j * D + i] : gIn[e]) : 0.0f;
    }
    __syncthreads();
    float lamBK = sPw[BK];

    int ib0 = 0;     // pre-pass: skip blocks whose decay weights are below 2^-skip_bits
    if (STATE_ONLY && a.skip_bits > 0.f && lam < 1.0f) {
        const float reach = a.skip_bits / -log2f(lam);
        if (reach < (float)(nblk * BK)) ib0 = max(0, nblk - ((int)(reach / BK) + 2));
    }
    for (int ib = ib0; ib < nblk; ++ib) {
        const int blk = rev ? (nblk - 1 - ib) : ib;
        const int t0 = seg_lo + blk * BK;
        // ---- load tiles (rows past the segment end are zero) ----
        for (int e = tid; e < BK * (D / 4); e += 256) {
            int r = e / (D / 4), c4 = (e % (D / 4)) * 4;
            int t = t0 + r;
            float4 vb = make_float4(0.f, 0.f, 0.f, 0.f), vc = vb, va = vb;
            if (t < seg_hi) {
                vb = *(const float4 *)(gB + (size_t)t * ldB + c4);
                vc = *(const float4 *)(gC + (size_t)t * ldC + c4);
                if (!STATE_ONLY) va = *(const float4 *)(gA + (size_t)t * ldA + c4);
                // Swish prologue on the operands that are pre-activations
                if (a.act & LA_ACT_BM) vb = make_float4(la_swish(vb.x), la_swish(vb.y), la_swish(vb.z), la_swish(vb.w));
                if (a.act & LA_ACT_C) vc = make_float4(la_swish(vc.x), la_swish(vc.y), la_swish(vc.z), la_swish(vc.w));
                if (!STATE_ONLY && (a.act & LA_ACT_A))
                    va = make_float4(la_swish(va.x), la_swish(va.y), la_swish(va.z), la_swish(va.w));
            }
            float *pb = sB + r * LD + c4, *pc = sC + r * LD + c4, *pa = sA + r * LD + c4;
            pb[0] = vb.x; pb[1] = vb.y; pb[2] = vb.z; pb[3] = vb.w;
            pc[0] = vc.x; pc[1] = vc.y; pc[2] = vc.z; pc[3] = vc.w;
            if (!STATE_ONLY) { pa[0] = va.x; pa[1] = va.y; pa[2] = va.z; pa[3] = va.w; }
        }
        __syncthreads();

        if (!STATE_ONLY) {
            // ---- masked scores S = (A Bm^T) * M ----
            float acc[RI][RI];
#pragma unroll
            for (int i = 0; i < RI; ++i)
#pragma unroll
                for (int j = 0; j < RI; ++j) acc[i][j] = 0.f;
            for (int k = 0; k < D; ++k) {
                float av[RI], bv[RI];
#pragma unroll
                for (int i = 0; i < RI; ++i) av[i] = sA[(ty + 16 * i) * LD + k];
#pragma unroll
                for (int j = 0; j < RI; ++j) bv[j] = sB[(tx + 16 * j) * LD + k];
#pragma unroll
                for (int i = 0; i < RI; ++i)
#pragma unroll
                    for (int j = 0; j < RI; ++j) acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
            }
#pragma unroll
            for (int i = 0; i < RI; ++i)
#pragma unroll
                for (int j = 0; j < RI; ++j) {
                    int r = ty + 16 * i, c = tx + 16 * j;
                    float m;
                    if (!REV) m = (r >= c) ? sPw[r - c] : 0.f;
                    else      m = (c >= r) ? sPw[c - r] : 0.f;
                    sS[r * LS + c] = acc[i][j] * m;
                }
            __syncthreads();

            // ---- Out = S C + rowscale * (A St) ----
            float oi[RI][CJ], ox[RI][CJ];
#pragma unroll
            for (int i = 0; i < RI; ++i)
#pragma unroll
                for (int j = 0; j < CJ; ++j) { oi[i][j] = 0.f; ox[i][j] = 0.f; }
            for (int c = 0; c < BK; ++c) {
                float sv[RI], cv[CJ];
#pragma unroll
                for (int i = 0; i < RI; ++i) sv[i] = sS[(ty + 16 * i) * LS + c];
#pragma unroll
                for (int j = 0; j < CJ; ++j) cv[j] = sC[c * LD + tx + 16 * j];
#pragma unroll
                for (int i = 0; i < RI; ++i)
#pragma unroll
                    for (int j = 0; j < CJ; ++j) oi[i][j] = fmaf(sv[i], cv[j], oi[i][j]);
            }
            for (int k = 0; k < D; ++k) {
                float av[RI], sv[CJ];
#pragma unroll
                for (int i = 0; i < RI; ++i) av[i] = sA[(ty + 16 * i) * LD + k];
#pragma unroll
                for (int j = 0; j < CJ; ++j) sv[j] = sKV[k * LD + tx + 16 * j];
#pragma unroll
                for (int i = 0; i < RI; ++i)
#pragma unroll
                    for (int j = 0; j < CJ; ++j) ox[i][j] = fmaf(av[i], sv[j], ox[i][j]);
            }
#pragma unroll
            for (int i = 0; i < RI; ++i) {
                int r = ty + 16 * i;
                int t = t0 + r;
                float rs = REV ? sPw[BK - r] : sPw[r + 1];
                if (t < seg_hi) {
#pragma unroll
                    for (int j = 0; j < CJ; ++j)
                    {
                        float o = fmaf(rs, ox[i][j], oi[i][j]);
                        if (a.act & LA_ACT_OUT) o *= la_swish_grad(gE[(size_t)t * ldE + tx + 16 * j]);
                        if (a.act & LA_ACT_ACC) o += gO[(size_t)t * ldO + tx + 16 * j];
                        gO[(size_t)t * ldO + tx + 16 * j] = o;
                    }
                }
            }
            __syncthreads();   // everyone is done reading the old state
        }

        // ---- St <- lambda^BK St + sum_r w_r Bm[r] C[r]^T ----
        // (when the final state is handed back, the last, partial block of m rows is
        //  weighted lambda^(m-1-r) and decays the old state by lambda^m)
        const int m_rows = (want_final && t0 + BK > seg_hi) ? seg_hi - t0 : BK;
        if (m_rows < BK) lamBK = sPw[m_rows];
        {
            float up[CJ][CJ];
#pragma unroll
            for (int i = 0; i < CJ; ++i)
#pragma unroll
                for (int j = 0; j < CJ; ++j) up[i][j] = 0.f;
            for (int r = 0; r < BK; ++r) {
                float w = rev ? sPw[r] : sPw[max(m_rows - 1 - r, 0)];
                float bv[CJ], cv[CJ];
#pragma unroll
                for (int i = 0; i < CJ; ++i) bv[i] = w * sB[r * LD + ty + 16 * i];
#pragma unroll
                for (int j = 0; j < CJ; ++j) cv[j] = sC[r * LD + tx + 16 * j];
#pragma unroll
                for (int i = 0; i < CJ; ++i)
#pragma unroll
                    for (int j = 0; j < CJ; ++j) up[i][j] = fmaf(bv[i], cv[j], up[i][j]);
            }
#pragma unroll
            for (int i = 0; i < CJ; ++i)
#pragma unroll
                for (int j = 0; j < CJ; ++j) {
                    float *p = sKV + (ty + 16 * i) * LD + tx + 16 * j;
                    *p = fmaf(lamBK, *p, up[i][j]);
                }
        }
        __syncthreads();
    }

    if (STATE_ONLY || want_final) {
        float *dst = STATE_ONLY ? gSt : a.st_out + (size_t)scan * (D * D);
        for (int e = tid; e < D * D; e += 256) {
            int i = e / D, j = e % D;
            dst[e] = sKV[i * LD + j];
        }
    }
}
