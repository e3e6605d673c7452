// grad_kernel: the two backward passes that contract the bucket statistics over the head dimension.
//
//   SIDE 0 (dQ), left to right, statistics S = (B | A) of (phi_K, [V | 1]) before/with token i:
//       dphi_Q(i)[r] = S[r,:] . [dO_i/e_i | -(dO_i.O_i)/e_i]
//   SIDE 1 (dK), right to left, statistics dS = (dB | dA) of (phi_Q, read-out cotangents) of tokens >= j:
//       dphi_K(j)[r] = dS[r,:] . [V_j | 1]
// followed in both cases by the chain rule through the corner softmax, tanh and W:  dx = W^T dz.
// "reader" is the tensor whose gradient is produced, "writer" the tensor that feeds the statistics.
//
// The statistics are held transposed, tiles S^T[head column][bucket row], so that a tile's accumulator
// registers are the B operand of the contraction over columns (lane = bucket row).  The in-tile part
// uses T^T[b][a] = Yw_b . Yr_a (+ the product of the two extra columns), masked to b <= a (b >= a
// right to left), whose accumulator is directly the A operand of  T . phi_writer.
#pragma once
#include "mfma_common.h"

namespace race {
namespace mfma {

// Developer aid: per-phase cycle counts of one workgroup (build with -DRACE_PHASE_TIMING).
#ifdef RACE_PHASE_TIMING
#define GRAD_PHASE_DECL long long ph_t[13] = {0}; long long ph_last = clock64();
#define GRAD_PHASE(i) { long long now_ = clock64(); ph_t[i] += now_ - ph_last; ph_last = now_; }
#define GRAD_PHASE_PRINT() if (blockIdx.x == 1 && blockIdx.y == 0 && (threadIdx.x & 63) == 0) \
    printf("grad side %d wave %d tiles %d: load %lld prod %lld tt %lld dP %lld upd %lld dphiw %lld smbwd %lld dX %lld | waits %lld %lld %lld %lld %lld\n", SIDE, (int)(threadIdx.x >> 6), ntiles, \
           ph_t[0], ph_t[2], ph_t[4], ph_t[5], ph_t[6], ph_t[8], ph_t[10], ph_t[12], ph_t[1], ph_t[3], ph_t[7], ph_t[9], ph_t[11]);
#else
#define GRAD_PHASE_DECL
#define GRAD_PHASE(i)
#define GRAD_PHASE_PRINT()
#endif

template <class C>
struct GradLds {
    static constexpr int wp = 0;                                        // [LPP][XS] bf16
    static constexpr int wpt = wp + C::LPP * C::XS * 2;                 // [D][ZS] bf16: W^T
    static constexpr int dz = wpt + C::D * C::ZS * 2;                   // [32][ZS] bf16
    static constexpr int sr = dz + kTile * C::ZS * 2;                   // [32] fp32 extra column of reader-Y
    static constexpr int sw = sr + kTile * 4;                           // [32] fp32 extra column of writer-Y
    static constexpr int area = (sw + kTile * 4 + 255) & ~255;
    // phase A
    static constexpr int xr = area;                                     // [32][XS]
    static constexpr int xw = xr + kTile * C::XS * 2;
    static constexpr int yr = xw + kTile * C::XS * 2;                   // reader-Y rows
    static constexpr int yw = yr + kTile * C::XS * 2;                   // writer-Y rows
    static constexpr int phw = yw + kTile * C::XS * 2;                  // [32][PS] writer assignments
    static constexpr int endA = phw + kTile * C::PS * 2;
    // phase B
    static constexpr int DS = C::LR + 4;                                // fp32 row stride
    static constexpr int dphi = area;                                   // [32][DS] fp32
    static constexpr int endB = dphi + kTile * DS * 4;
    static constexpr int total = endA > endB ? endA : endB;
    static_assert(total <= 160 * 1024, "LDS budget");
};

template <class C, int SIDE>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(1, 1)))
void grad_kernel(KArgs a, const bf16raw *Q, const bf16raw *K, const bf16raw *V, const bf16raw *O,
                 const float *den, const bf16raw *dO, bf16raw *dX)
{
    using S = GradLds<C>;
    extern __shared__ __attribute__((aligned(256))) unsigned char lds[];
    bf16raw *wp = reinterpret_cast<bf16raw *>(lds + S::wp);
    bf16raw *wpt = reinterpret_cast<bf16raw *>(lds + S::wpt);
    bf16raw *dz = reinterpret_cast<bf16raw *>(lds + S::dz);
    float *sr = reinterpret_cast<float *>(lds + S::sr);
    float *sw = reinterpret_cast<float *>(lds + S::sw);
    bf16raw *xr = reinterpret_cast<bf16raw *>(lds + S::xr);
    bf16raw *xw = reinterpret_cast<bf16raw *>(lds + S::xw);
    bf16raw *yr = reinterpret_cast<bf16raw *>(lds + S::yr);
    bf16raw *yw = reinterpret_cast<bf16raw *>(lds + S::yw);
    bf16raw *phw = reinterpret_cast<bf16raw *>(lds + S::phw);
    float *dphi = reinterpret_cast<float *>(lds + S::dphi);

    constexpr bool kReverse = (SIDE == 1);
    const int seg = blockIdx.x, bh = blockIdx.y, head = bh % a.H;
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, ln = lane & 31, h = lane >> 5;
    const int r_own = w * C::LRW;
    const bool intra = a.causal;

    const size_t base = static_cast<size_t>(bh) * a.N * C::D;
    Q += base; K += base; V += base; O += base; dO += base; dX += base;
    den += static_cast<size_t>(bh) * a.N;
    const bf16raw *Xr = SIDE == 0 ? Q : K, *Xw = SIDE == 0 ? K : Q;
    const float *st = a.state + (static_cast<size_t>(bh) * a.nseg + seg) * C::STATE;

    {
        const bf16raw *src = a.Wp + static_cast<size_t>(head) * C::LPP * C::D;
        for (int c = tid; c < C::LPP * C::CPR; c += kThreads) {
            const int row = c / C::CPR, ch = c % C::CPR;
            *reinterpret_cast<u32x4 *>(wp + row * C::XS + ch * 8) = *reinterpret_cast<const u32x4 *>(src + row * C::D + ch * 8);
        }
        const bf16raw *srct = a.WpT + static_cast<size_t>(head) * C::D * C::LPP;
        for (int c = tid; c < C::D * (C::LPP / 8); c += kThreads) {
            const int row = c / (C::LPP / 8), ch = c % (C::LPP / 8);
            *reinterpret_cast<u32x4 *>(wpt + row * C::ZS + ch * 8) = *reinterpret_cast<const u32x4 *>(srct + row * C::LPP + ch * 8);
        }
    }
    // statistics at the start of the segment, transposed tiles: ST[column tile][bucket-row tile]
    f32x16 ST[C::NT][C::MT];
    float macc[C::MT];          // extra column (A or dA): per-half partial sums, lane n <-> row r_own + 32*ntc + n
#pragma unroll
    for (int ntc = 0; ntc < C::MT; ++ntc) {
#pragma unroll
        for (int mtc = 0; mtc < C::NT; ++mtc) {
#pragma unroll
            for (int v = 0; v < 16; ++v)
                ST[mtc][ntc][v] = st[(r_own + 32 * ntc + ln) * C::D + 32 * mtc + acc_row(v, h)];
        }
        macc[ntc] = (h == 0) ? st[C::LR * C::D + r_own + 32 * ntc + ln] : 0.f;
    }

    const int64_t t_begin = seg * a.seg_len;
    const int64_t t_end = (t_begin + a.seg_len < a.N) ? t_begin + a.seg_len : a.N;
    const int ntiles = static_cast<int>((t_end - t_begin + kTile - 1) / kTile);

    auto tile_t0 = [&](int it) { return t_begin + static_cast<int64_t>(kReverse ? ntiles - 1 - it : it) * kTile; };
    auto tile_nv = [&](int64_t t0) { return (t_end - t0 < kTile) ? static_cast<int>(t_end - t0) : kTile; };

    // loads run one tile ahead of the arithmetic
    RowChunks<C> pre_r, pre_w, pre_v;
    CotChunks<C> pre_c;
    auto fetch = [&](int it) {
        const int64_t t0 = tile_t0(it);
        const int nv = tile_nv(t0);
        fetch_rows<C>(Xr, t0, nv, pre_r);
        if (intra) fetch_rows<C>(Xw, t0, nv, pre_w);
        if (SIDE == 1 || intra) fetch_rows<C>(V, t0, nv, pre_v);
        if (SIDE == 0 || intra) fetch_cotangent<C>(dO, O, den, t0, nv, pre_c);
    };
#ifdef RACE_GRAD_PREFETCH
    if (ntiles > 0) fetch(0);
#endif

    GRAD_PHASE_DECL
    for (int it = 0; it < ntiles; ++it) {
        const int64_t t0 = tile_t0(it);
        const int nvalid = tile_nv(t0);

        // ---- registers -> LDS
#ifndef RACE_GRAD_PREFETCH
        fetch(it);
#endif
        store_rows<C>(pre_r, xr);
        if (intra) store_rows<C>(pre_w, xw);
        if (SIDE == 0) {
            store_cotangent<C>(pre_c, yr, sr);
            if (intra) store_rows<C>(pre_v, yw);
            if (tid < kTile) sw[tid] = 1.f;
        } else {
            store_rows<C>(pre_v, yr);
            if (intra) store_cotangent<C>(pre_c, yw, sw);
            if (tid < kTile) sr[tid] = 1.f;
        }
        GRAD_PHASE(0)
        __syncthreads();
        GRAD_PHASE(1)

        // ---- production
        const int side = w / C::NG, g = w % C::NG;
        f32x16 z = {0};
        if (side == 0) {
            z = project<C>(wp, xr, g, ln, h);
        } else if (side == 1 && intra) {
            const f32x16 zw = project<C>(wp, xw, g, ln, h);
            write_assignments<C>(zw, g, ln, h, a.beta, ln < nvalid, phw);
        }
        GRAD_PHASE(2)
        __syncthreads();
        GRAD_PHASE(3)

        // ---- in-tile part: T^T[b][a] = Yw_b . Yr_a + sw_b * sr_a, masked
        f32x16 tt = {0};
        if (intra) {
#pragma unroll
            for (int s = 0; s < C::D / 16; ++s) {
                const u32x4 aw = lds128(yw + ln * C::XS + 16 * s + 8 * h);
                const u32x4 br = lds128(yr + ln * C::XS + 16 * s + 8 * h);
                tt = mma(aw, br, tt);
            }
            const float sra = sr[ln];
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int b = acc_row(v, h);
                const bool keep = kReverse ? (b >= ln) : (b <= ln);
                tt[v] = keep ? fmaf(sw[b], sra, tt[v]) : 0.f;
            }
        }
        GRAD_PHASE(4)
        // ---- cotangent of the reader's assignments for this wavefront's bucket rows
        f32x16 dP[C::MT];
#pragma unroll
        for (int ntc = 0; ntc < C::MT; ++ntc) dP[ntc] = f32x16{0};
#pragma unroll
        for (int mtc = 0; mtc < C::NT; ++mtc) {
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const int cc = 32 * mtc + 16 * s + 4 * h;
                const u32x4 ay = lds64x2(yr + ln * C::XS + cc, yr + ln * C::XS + cc + 8);
#pragma unroll
                for (int ntc = 0; ntc < C::MT; ++ntc) dP[ntc] = mma(ay, acc_operand(ST[mtc][ntc], s), dP[ntc]);
                RACE_SCHED_FENCE();
            }
        }
        if (intra) {
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const u32x4 at = acc_operand(tt, s);
#pragma unroll
                for (int ntc = 0; ntc < C::MT; ++ntc)
                    dP[ntc] = mma(at, lds_tr_acc(phw, C::PS, 16 * s, r_own + 32 * ntc, ln, h), dP[ntc]);
            }
        }
        {
            // extra column: + sr_a * (A or dA)[r] with the masses before this tile
            float srv[16];
#pragma unroll
            for (int v = 0; v < 16; ++v) srv[v] = sr[acc_row(v, h)];
#pragma unroll
            for (int ntc = 0; ntc < C::MT; ++ntc) {
                const float m = macc[ntc] + __shfl_xor(macc[ntc], 32, 64);
#pragma unroll
                for (int v = 0; v < 16; ++v) dP[ntc][v] = fmaf(srv[v], m, dP[ntc][v]);
            }
        }
        GRAD_PHASE(5)
        // ---- statistics += Yw^T . phi_writer
        if (intra) {
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                u32x4 ya[C::NT];
#pragma unroll
                for (int mtc = 0; mtc < C::NT; ++mtc) ya[mtc] = lds_tr_plain(yw, C::XS, 16 * s, 32 * mtc, ln, h);
                float gw[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) gw[e] = sw[16 * s + 8 * h + e];
#pragma unroll
                for (int ntc = 0; ntc < C::MT; ++ntc) {
                    const u32x4 bp = lds_tr_plain(phw, C::PS, 16 * s, r_own + 32 * ntc, ln, h);
                    macc[ntc] += bf_lo(bp.x) * gw[0] + bf_hi(bp.x) * gw[1] + bf_lo(bp.y) * gw[2] + bf_hi(bp.y) * gw[3] +
                                 bf_lo(bp.z) * gw[4] + bf_hi(bp.z) * gw[5] + bf_lo(bp.w) * gw[6] + bf_hi(bp.w) * gw[7];
#pragma unroll
                    for (int mtc = 0; mtc < C::NT; ++mtc) ST[mtc][ntc] = mma(ya[mtc], bp, ST[mtc][ntc]);
                    RACE_SCHED_FENCE();
                }
            }
        }
        GRAD_PHASE(6)
        __syncthreads();        // phase-A tiles are dead from here on
        GRAD_PHASE(7)

        // ---- hand the cotangents to the lanes that own (token, table)
#pragma unroll
        for (int ntc = 0; ntc < C::MT; ++ntc) {
#pragma unroll
            for (int v = 0; v < 16; ++v) dphi[acc_row(v, h) * S::DS + r_own + 32 * ntc + ln] = dP[ntc][v];
        }
        // the next tile's loads fly during the vector-ALU phases below (few registers are live here)
#ifdef RACE_GRAD_PREFETCH
        if (it + 1 < ntiles) fetch(it + 1);
#endif
        GRAD_PHASE(8)
        __syncthreads();
        GRAD_PHASE(9)

        // ---- back through the corner softmax and tanh (Algorithm 1, step 4):
        //      with w_r = phi_r dphi_r, m = sum_r w_r, E_t = sum_r v_{r,t} w_r:
        //      du_t = beta (E_t - m (p_t - q_t)),  dz_t = du_t (1 - tanh^2 z_t)
        if (side == 0) {
            float dzv[16];
#pragma unroll
            for (int v = 0; v < 16; ++v) dzv[v] = 0.f;
#pragma unroll
            for (int j = 0; j < C::TPL; ++j) {
                const int table = g * C::TPG + h * C::TPL + j;
                if (table >= C::L) break;
                float p[C::P], q[C::P], sech2[C::P], lo[1 << C::PLO], hi[1 << C::PHI];
                bit_masses<C>(z, j, a.beta, p, q, sech2);
                kron_factors<C>(p, q, lo, hi);
                float E[C::P];
#pragma unroll
                for (int t = 0; t < C::P; ++t) E[t] = 0.f;
                float m = 0.f;
                float chunk[1 << C::PHI];
#pragma unroll
                for (int aa = 0; aa < (1 << C::PHI); ++aa) {
                    const float *src = dphi + ln * S::DS + table * C::R + aa * 8;
                    const float4 d0 = *reinterpret_cast<const float4 *>(src);
                    const float4 d1 = *reinterpret_cast<const float4 *>(src + 4);
                    const float wv[8] = {hi[aa] * lo[0] * d0.x, hi[aa] * lo[1] * d0.y, hi[aa] * lo[2] * d0.z, hi[aa] * lo[3] * d0.w,
                                         hi[aa] * lo[4] * d1.x, hi[aa] * lo[5] * d1.y, hi[aa] * lo[6] * d1.z, hi[aa] * lo[7] * d1.w};
                    const float s01 = wv[0] + wv[1], s23 = wv[2] + wv[3], s45 = wv[4] + wv[5], s67 = wv[6] + wv[7];
                    E[0] += ((wv[1] - wv[0]) + (wv[3] - wv[2])) + ((wv[5] - wv[4]) + (wv[7] - wv[6]));
                    if (C::PLO > 1) E[1] += (s23 - s01) + (s67 - s45);
                    const float s0123 = s01 + s23, s4567 = s45 + s67;
                    if (C::PLO > 2) E[2] += s4567 - s0123;
                    chunk[aa] = s0123 + s4567;
                }
#pragma unroll
                for (int aa = 0; aa < (1 << C::PHI); ++aa) {
                    m += chunk[aa];
#pragma unroll
                    for (int t = 0; t < C::PHI; ++t) E[C::PLO + t] += ((aa >> t) & 1) ? chunk[aa] : -chunk[aa];
                }
#pragma unroll
                for (int t = 0; t < C::P; ++t)
                    dzv[zslot<C>(j, t)] = a.beta * (E[t] - m * (p[t] - q[t])) * sech2[t];
            }
            // register v of the projection accumulator is projection row acc_row(v, h) of group g
#pragma unroll
            for (int aa = 0; aa < 4; ++aa) {
                *reinterpret_cast<u32x2 *>(dz + ln * C::ZS + g * 32 + 8 * aa + 4 * h) =
                    u32x2{pack2(dzv[4 * aa], dzv[4 * aa + 1]), pack2(dzv[4 * aa + 2], dzv[4 * aa + 3])};
            }
        }
        GRAD_PHASE(10)
        __syncthreads();
        GRAD_PHASE(11)

        // ---- dX = dZ . W
        for (int nt = w; nt < C::NT; nt += kWaves) {
            f32x16 acc = {0};
#pragma unroll
            for (int s = 0; s < C::LPP / 16; ++s) {
                const u32x4 az = lds128(dz + ln * C::ZS + 16 * s + 8 * h);
                const u32x4 bw = lds128(wpt + (32 * nt + ln) * C::ZS + 16 * s + 8 * h);
                acc = mma(az, bw, acc);
            }
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = acc_row(v, h);
                if (row < nvalid) dX[(t0 + row) * C::D + 32 * nt + ln] = static_cast<bf16raw>(pack2(acc[v], 0.f) & 0xffffu);
            }
        }
        GRAD_PHASE(12)
        __syncthreads();
        GRAD_PHASE(1)
    }
    GRAD_PHASE_PRINT()
}

}  // namespace mfma
}  // namespace race
