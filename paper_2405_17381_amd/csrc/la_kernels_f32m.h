// fp32 path on the matrix cores: the block loop of Alg. 5 / Alg. 6 with every
// contraction on v_mfma_f32_32x32x2_f32 (fp32 operands, fp32 accumulation: no
// rounding below fp32 anywhere).  Used for d = 128; blocks of BK = 32 rows.
//
// One workgroup of D/32 wavefronts per (scan, segment).  Wave w owns the value-
// feature slice j in [32w, 32w+32): its columns of Out and of the state
// St[:, slice], which lives in accumulator registers for the whole segment.
// Per block:
//   scores  S[q][key] = sum_f A[q][f] Bm[key][f]: one 32x32 tile; the feature sum is
//           split over the waves (32 features each), partial tiles go to LDS, and
//           every wave adds them up (x decay mask) into its own operand registers
//   inter   Out[q][j]  = scale(q) sum_i A[q][i] St[i][j]     state operand straight
//           from the accumulator registers (register v of tile mt is row
//           32 mt + 8 (v/4) + 4 (lane/32) + v%4: as the k-th operand element of
//           lane/32 it pairs rows i and i+4, and the A tile is read to match)
//   intra   Out[q][j] += sum_key P[q][key] C[key][j]
//   update  St[i][j]   = lambda^BK St[i][j] + sum_r w_r Bm[r][i] C[r][j]
// MFMA 32x32x2 f32 layout (lane l): A operand = A[l%32][l/32], B operand =
// B[l/32][l%32], C/D: column l%32, register v = row 8 (v/4) + 4 (l/32) + v%4.
// Operands are single floats read from row-major LDS tiles (row stride D+1:
// conflict free for both the row-wise and the column-wise walks), so transposes
// cost nothing.  The next block's tiles are prefetched into registers.
#pragma once
#include "la_common.h"

typedef float f32m_x16 __attribute__((ext_vector_type(16)));

template <int D>
struct F32mCfg {
    static constexpr int BK = 32;
    static constexpr int NW = D / 32;
    static constexpr int NT = NW * 64;
    static constexpr int LD = D + 1;                 // row stride of the A, Bm, C tiles (floats)
    static constexpr int LSP = BK + 1;               // row stride of the partial score tiles
    static constexpr int NV = BK * (D / 4) / NT;     // float4 loads per thread per tile (= 4)
    static constexpr size_t lds_bytes = sizeof(float) * (size_t)(3 * BK * LD + NW * BK * LSP + (2 * BK + 1));
};

// LDS loads of a batch are issued before the MFMAs that use them and may not cross
#define LA_F32M_FENCE() __builtin_amdgcn_sched_barrier(0x476)

__device__ __forceinline__ f32m_x16 mfma_f32(float a, float b, f32m_x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

template <int D, bool REV, bool STATE_ONLY>
__global__ __launch_bounds__(D * 2, 2) void la_scan_f32m(ScanLaunch launch, LaLambdas lams)
{
    using Cfg = F32mCfg<D>;
    constexpr int BK = Cfg::BK, NW = Cfg::NW, NT = Cfg::NT, LD = Cfg::LD, LSP = Cfg::LSP, NV = Cfg::NV;
    constexpr int MT_D = D / 32;

    // two roles (two independent pre-passes in one launch) follow one another in the grid
    const int role = launch.nroles == 2 ? (int)(blockIdx.x / launch.items) : 0;
    const int item = launch.nroles == 2 ? (int)(blockIdx.x % launch.items) : (int)blockIdx.x;
    const ScanArgs &a = launch.r[role];

    extern __shared__ float smem_f32m[];
    float *sA = smem_f32m;
    float *sB = sA + BK * LD;
    float *sC = sB + BK * LD;
    float *sSp = sC + BK * LD;                       // [NW][BK][LSP]
    // lambda^k for k = 0..BK at sPw[k]; sPw[-BK..-1] = 0, so that the weight lambda^(m-1-r) of a
    // row r >= m of a final, partial block (the row itself is zero) is read without a clamp
    float *sPw = sSp + NW * BK * LSP + BK;

    const int tid = threadIdx.x;
    const int w = tid >> 6, l = tid & 63, l32 = l & 31, g = l >> 5;
    const int seg = item % a.S;
    int scan = item / a.S;
    if (STATE_ONLY) {
        const int b = scan % a.B, hd = scan / a.B;   // heads in dispatch order
        scan = b * a.H + lams.order[hd];
    }
    const float lam = lams.v[scan % a.H];
    const bool rev = STATE_ONLY ? (a.rev != 0) : REV;
    if (STATE_ONLY) {
        if (!rev && seg == a.S - 1) return;          // never consumed
        if (rev && seg == 0) return;
    }
    const int seg_lo = seg * a.L;
    const int seg_hi = min(a.n, seg_lo + a.L);
    const int nblk = (seg_hi - seg_lo + BK - 1) / BK;

    const int bi = scan / a.H, hi = scan % a.H;
    const float *gA = (const float *)a.A + (size_t)bi * a.lA.bs + (size_t)hi * a.lA.hs;
    const float *gB = (const float *)a.Bm + (size_t)bi * a.lB.bs + (size_t)hi * a.lB.hs;
    const float *gC = (const float *)a.C + (size_t)bi * a.lC.bs + (size_t)hi * a.lC.hs;
    float *gO = (float *)a.Out + (size_t)bi * a.lO.bs + (size_t)hi * a.lO.hs;
    const float *gE = (a.act & LA_ACT_OUT) ? (const float *)a.E + (size_t)bi * a.lE.bs + (size_t)hi * a.lE.hs : gA;
    const int ldA = a.lA.ld, ldB = a.lB.ld, ldC = a.lC.ld, ldO = a.lO.ld, ldE = a.lE.ld;
    float *gSt = a.states ? a.states + ((size_t)scan * a.S + seg) * (size_t)(D * D) : nullptr;

    // lambda^k, evaluated in double then rounded once
    for (int k = tid - BK; k <= BK; k += NT) sPw[k] = k < 0 ? 0.0f : (float)pow((double)lam, (double)k);

    // ---- running state St[i][j], j = 32 w + l32, in accumulator layout -----------------------
    f32m_x16 st[MT_D];
    const float *gIn = STATE_ONLY ? nullptr : la_entering_state(a, scan, seg, REV, lams.lg2[scan % a.H], D * D);
#pragma unroll
    for (int mt = 0; mt < MT_D; ++mt)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int i = 32 * mt + 8 * (v >> 2) + 4 * g + (v & 3), j = 32 * w + l32;
            st[mt][v] = gIn ? (a.transpose_init ? gIn[(size_t)j * D + i] : gIn[(size_t)i * D + j]) : 0.0f;
        }
    const bool want_final = !STATE_ONLY && !REV && a.st_out != nullptr && seg == a.S - 1;

    int ib0 = 0;     // pre-pass: skip blocks whose decay weights are below 2^-skip_bits
    if (STATE_ONLY && a.skip_bits > 0.f && lam < 1.0f) {
        const float reach = a.skip_bits / -log2f(lam);
        if (reach < (float)(nblk * BK)) ib0 = max(0, nblk - ((int)(reach / BK) + 2));
    }
    __syncthreads();                                 // sPw ready

    // ---- global -> register prefetch (rows past the segment end read the last row; they are
    // zeroed when the block is staged) -----------------------------------------------------------
    float4 ra[NV], rb[NV], rc[NV];
    auto load_block = [&](int blk) {
        const int t0 = seg_lo + blk * BK;
#pragma unroll
        for (int u = 0; u < NV; ++u) {
            const int e = tid + u * NT;
            const int r = e / (D / 4), c4 = (e % (D / 4)) * 4;
            const size_t row = (size_t)min(t0 + r, seg_hi - 1);
            rb[u] = *(const float4 *)(gB + row * ldB + c4);
            rc[u] = *(const float4 *)(gC + row * ldC + c4);
            if (!STATE_ONLY) ra[u] = *(const float4 *)(gA + row * ldA + c4);
        }
    };
    auto act4 = [](float4 x) { return make_float4(la_swish(x.x), la_swish(x.y), la_swish(x.z), la_swish(x.w)); };
    auto stage_block = [&](int t0) {
#pragma unroll
        for (int u = 0; u < NV; ++u) {
            const int e = tid + u * NT;
            const int r = e / (D / 4), c4 = (e % (D / 4)) * 4;
            const bool ok = t0 + r < seg_hi;
            const float4 z = make_float4(0.f, 0.f, 0.f, 0.f);
            float4 vb = ok ? rb[u] : z, vc = ok ? rc[u] : z, va = (!STATE_ONLY && ok) ? ra[u] : z;
            if (a.act & LA_ACT_BM) vb = act4(vb);
            if (a.act & LA_ACT_C) vc = act4(vc);
            if (!STATE_ONLY && (a.act & LA_ACT_A)) va = act4(va);
            float *pb = sB + r * LD + c4, *pc = sC + r * LD + c4;
            pb[0] = vb.x; pb[1] = vb.y; pb[2] = vb.z; pb[3] = vb.w;
            pc[0] = vc.x; pc[1] = vc.y; pc[2] = vc.z; pc[3] = vc.w;
            if (!STATE_ONLY) {
                float *pa = sA + r * LD + c4;
                pa[0] = va.x; pa[1] = va.y; pa[2] = va.z; pa[3] = va.w;
            }
        }
    };

    if (ib0 < nblk) load_block(rev ? nblk - 1 - ib0 : ib0);

    for (int ib = ib0; ib < nblk; ++ib) {
        const int blk = rev ? (nblk - 1 - ib) : ib;
        const int t0 = seg_lo + blk * BK;
        stage_block(t0);
        if (ib + 1 < nblk) load_block(rev ? blk - 1 : blk + 1);
        __syncthreads();                             // tiles staged

        // this wave's C operands, row r = 2 ks + g: shared by the intra product and the update
        float cfrag[16];
#pragma unroll
        for (int ks = 0; ks < 16; ++ks) cfrag[ks] = sC[(2 * ks + g) * LD + 32 * w + l32];

        if (!STATE_ONLY) {
            // ---- partial scores over this wave's 32 features ------------------------------------
            {
                f32m_x16 s = {0};
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    float fa[8], fb[8];
#pragma unroll
                    for (int k = 0; k < 8; ++k) {
                        const int f = 32 * w + 2 * (8 * h + k) + g;
                        fa[k] = sA[l32 * LD + f];
                        fb[k] = sB[l32 * LD + f];
                    }
                    LA_F32M_FENCE();
#pragma unroll
                    for (int k = 0; k < 8; ++k) s = mfma_f32(fa[k], fb[k], s);
                }
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int q = 8 * (v >> 2) + 4 * g + (v & 3);
                    sSp[(w * BK + q) * LSP + l32] = s[v];
                }
            }
            // ---- inter block: acc[q][j] = scale(q) sum_i A[q][i] St[i][j] -------------------------
            f32m_x16 acc = {0};
#pragma unroll
            for (int mt = 0; mt < MT_D; ++mt)
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    float fa[8];
#pragma unroll
                    for (int k = 0; k < 8; ++k) {
                        const int v = 8 * h + k;
                        fa[k] = sA[l32 * LD + 32 * mt + 8 * (v >> 2) + 4 * g + (v & 3)];
                    }
                    LA_F32M_FENCE();
#pragma unroll
                    for (int k = 0; k < 8; ++k) acc = mfma_f32(fa[k], st[mt][8 * h + k], acc);
                }
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int q = 8 * (v >> 2) + 4 * g + (v & 3);
                acc[v] *= REV ? sPw[BK - q] : sPw[q + 1];
            }
            __syncthreads();                         // partial score tiles complete
            // ---- intra block: acc[q][j] += sum_key P[q][key] C[key][j] ----------------------------
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                float p[8];
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    const int key = 2 * (8 * h + k) + g, q = l32;
                    float x = 0.f;
#pragma unroll
                    for (int ww = 0; ww < NW; ++ww) x += sSp[(ww * BK + q) * LSP + key];
                    const int dist = REV ? key - q : q - key;
                    p[k] = dist >= 0 ? x * sPw[dist] : 0.f;
                }
                LA_F32M_FENCE();
#pragma unroll
                for (int k = 0; k < 8; ++k) acc = mfma_f32(p[k], cfrag[8 * h + k], acc);
            }
            // ---- store (epilogue: phi' of the pre-activation tile, or add to what is there) -------
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int q = 8 * (v >> 2) + 4 * g + (v & 3);
                const int t = t0 + q;
                if (t < seg_hi) {
                    float o = acc[v];
                    if (a.act & LA_ACT_OUT) o *= la_swish_grad(gE[(size_t)t * ldE + 32 * w + l32]);
                    if (a.act & LA_ACT_ACC) o += gO[(size_t)t * ldO + 32 * w + l32];
                    gO[(size_t)t * ldO + 32 * w + l32] = o;
                }
            }
        }

        // ---- St <- lambda^BK St + sum_r w_r Bm[r] C[r]^T ----------------------------------------
        // (when the final state is handed back, the last, partial block of m rows is weighted
        //  lambda^(m-1-r) and decays the old state by lambda^m; its rows past m are zero)
        {
            const int m = (want_final && t0 + BK > seg_hi) ? seg_hi - t0 : BK;
            const float decay = sPw[m];
            float wgt[16];                           // weight of row r = 2 ks + g
#pragma unroll
            for (int ks = 0; ks < 16; ++ks) wgt[ks] = rev ? sPw[2 * ks + g] : sPw[m - 1 - (2 * ks + g)];
#pragma unroll
            for (int mt = 0; mt < MT_D; ++mt) {
                f32m_x16 s = st[mt];
#pragma unroll
                for (int v = 0; v < 16; ++v) s[v] *= decay;
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    float fb[8];
#pragma unroll
                    for (int k = 0; k < 8; ++k) {
                        const int ks = 8 * h + k;
                        fb[k] = wgt[ks] * sB[(2 * ks + g) * LD + 32 * mt + l32];
                    }
                    LA_F32M_FENCE();
#pragma unroll
                    for (int k = 0; k < 8; ++k) s = mfma_f32(fb[k], cfrag[8 * h + k], s);
                }
                st[mt] = s;
            }
        }
        __syncthreads();                             // every tile of this block is dead
    }

    if (STATE_ONLY || want_final) {
        // through LDS (every tile is dead by now), so that the copy to memory is a short loop of
        // 16-byte stores instead of 64 scattered ones per lane
        float *dst = STATE_ONLY ? gSt : a.st_out + (size_t)scan * (D * D);
        float *sKV = smem_f32m;                      // [D][D], D*D floats fit in the tiles' storage
#pragma unroll
        for (int mt = 0; mt < MT_D; ++mt)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int i = 32 * mt + 8 * (v >> 2) + 4 * g + (v & 3);
                sKV[i * D + 32 * w + l32] = st[mt][v];
            }
        __syncthreads();
#pragma unroll 1
        for (int e = tid * 4; e < D * D; e += NT * 4) *(float4 *)(dst + e) = *(const float4 *)(sKV + e);
    }
}
