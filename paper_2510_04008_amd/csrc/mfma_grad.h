// grad_kernel: the two backward passes that contract the bucket statistics over the head dimension.
// Register budget: with eight wavefronts of 256 registers a wavefront can carry 32 bucket rows x d
// columns of fp32 statistics next to its working set, i.e. 256 bucket rows per workgroup.  Shapes with
// more rows are split over TSPLIT workgroups by tables (blockIdx.z): each computes dz for its own
// tables and writes it to the workspace; dz_matmul_kernel then forms dX = dZ . W for all tables.
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
struct GradCfg {
    static constexpr int TSPLIT = C::LR / (32 * kWaves);                // workgroups per (segment, head)
    static constexpr int NGW = C::NG / TSPLIT;                          // projection groups per workgroup
    static constexpr int RW = kWaves / NGW;                             // wavefronts per projection group
    static constexpr int JW = C::TPL < RW ? C::TPL : RW;                // ... split over the lane's tables
    static constexpr int AW = RW / JW;                                  // ... and over the high-bit index
    static constexpr int AN = (1 << C::PHI) / AW;                       // high-bit indices per wavefront
    static constexpr int ROWS = C::LR / TSPLIT;                         // bucket rows per workgroup
    static_assert(TSPLIT >= 1 && C::NG % TSPLIT == 0 && kWaves % NGW == 0, "table split");
    static_assert(AW >= 1 && AN >= 1 && AN * AW == (1 << C::PHI), "assignment split");
    static_assert(NGW * C::TPG * C::R == ROWS, "a workgroup's rows are the tables of its projection groups");
    static_assert(AW == 1 || (C::TPL == JW && C::P <= 7), "the split backward pass handles one table per wavefront");
    static_assert(NGW * C::TPL <= kWaves && NGW + 1 <= kWaves, "production roles must fit the wavefronts");
};

template <class C>
struct GradLds {
    using G = GradCfg<C>;
    static constexpr int wp = 0;                                        // [LPP][XS] bf16
    static constexpr int DZS = G::NGW * 32 + 8;                         // bf16 row stride of the dz tile
    static constexpr int dz = wp + C::LPP * C::XS * 2;                  // [32][DZS] bf16
    static constexpr int sr = dz + kTile * DZS * 2;                     // [32] fp32 extra column of reader-Y
    static constexpr int sw = sr + kTile * 4;                           // [32] fp32 extra column of writer-Y
    static constexpr int zl = (sw + kTile * 4 + 15) & ~15;              // [NGW][64][16] fp32: reader projections
    static constexpr int yr = zl + G::NGW * 64 * 16 * 4;                // [32][XS] reader-Y rows
    static constexpr int ttop = yr + kTile * C::XS * 2;                 // [2][64] x 16 B: masked in-tile term as MFMA operands
    static constexpr int area = (ttop + 2 * 64 * 16 + 255) & ~255;
    // phase A
    static constexpr int xr = area;                                     // [32][XS]
    static constexpr int xw = xr + kTile * C::XS * 2;
    static constexpr int yw = xw + kTile * C::XS * 2;                   // writer-Y rows
    static constexpr int phw = yw + kTile * C::XS * 2;                  // [32][PS] writer assignments
    static constexpr int endA = phw + kTile * C::PS * 2;
    // phase B
    static constexpr int DS = G::ROWS + 4;                              // fp32 row stride
    static constexpr int dphi = area;                                   // [32][DS] fp32
    static constexpr int part = dphi + kTile * DS * 4;                  // [AW-1][NGW*JW][64][8] fp32: partial sums
    static constexpr int endB = part + (G::AW - 1) * G::NGW * G::JW * 64 * 8 * 4;
    static constexpr int total = endA > endB ? endA : endB;
    static_assert(total <= 160 * 1024, "LDS budget");
};

template <class C, int SIDE>
__global__ __launch_bounds__(kThreads)
void grad_kernel(KArgs a, const bf16raw *Q, const bf16raw *K, const bf16raw *V, const bf16raw *O,
                 const float *den, const bf16raw *dO, bf16raw *dZ)
{
    using S = GradLds<C>;
    using G = GradCfg<C>;
    extern __shared__ __attribute__((aligned(256))) unsigned char lds[];
    bf16raw *wp = reinterpret_cast<bf16raw *>(lds + S::wp);
    bf16raw *dz = reinterpret_cast<bf16raw *>(lds + S::dz);
    float *sr = reinterpret_cast<float *>(lds + S::sr);
    float *sw = reinterpret_cast<float *>(lds + S::sw);
    float *zl = reinterpret_cast<float *>(lds + S::zl);
    bf16raw *yr = reinterpret_cast<bf16raw *>(lds + S::yr);
    bf16raw *xr = reinterpret_cast<bf16raw *>(lds + S::xr);
    bf16raw *xw = reinterpret_cast<bf16raw *>(lds + S::xw);
    bf16raw *yw = reinterpret_cast<bf16raw *>(lds + S::yw);
    bf16raw *phw = reinterpret_cast<bf16raw *>(lds + S::phw);
    float *dphi = reinterpret_cast<float *>(lds + S::dphi);
    float *part = reinterpret_cast<float *>(lds + S::part);
    u32x4 *ttop = reinterpret_cast<u32x4 *>(lds + S::ttop);

    constexpr bool kReverse = (SIDE == 1);
    const int seg = blockIdx.x, bh = blockIdx.y, head = bh % a.H;
    const int tid = threadIdx.x, w = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, ln = lane & 31, h = lane >> 5;
    const int th = blockIdx.z;                       // which share of the tables this workgroup owns
    const int r_base = th * G::ROWS;                 // its first bucket row
    const int r_own = r_base + w * 32;               // this wavefront's 32 bucket rows
    // production share: projection group g; tables j = jq, jq + JW, ... of the lane; high-bit indices [a0, a0 + AN)
    const int gl = w % G::NGW, g = th * G::NGW + gl;
    const int jq = (w / G::NGW) % G::JW, aq = (w / G::NGW) / G::JW, a0 = aq * G::AN;
    const bool intra = a.causal;

    const size_t base = static_cast<size_t>(bh) * a.N * C::D;
    Q += base; K += base; V += base; O += base; dO += base;
    dZ += static_cast<size_t>(bh) * a.N * C::LPP;
    den += static_cast<size_t>(bh) * a.N;
    const bf16raw *Xr = SIDE == 0 ? Q : K, *Xw = SIDE == 0 ? K : Q;
    const float *st = a.state + (static_cast<size_t>(bh) * a.nseg + seg) * C::STATE;

    {
        const bf16raw *src = a.Wp + static_cast<size_t>(head) * C::LPP * C::D;
        for (int c = tid; c < C::LPP * C::CPR; c += kThreads) {
            const int row = c / C::CPR, ch = c % C::CPR;
            *reinterpret_cast<u32x4 *>(wp + row * C::XS + ch * 8) = *reinterpret_cast<const u32x4 *>(src + row * C::D + ch * 8);
        }
    }
    // statistics at the start of the segment, transposed tiles: ST[column tile][bucket-row tile]
    f32x16 ST[C::NT];         // ST[column tile]: columns x this wavefront's 32 bucket rows
    float macc;               // extra column (A or dA): per-half partial sum, lane n <-> row r_own + n
#pragma unroll
    for (int mtc = 0; mtc < C::NT; ++mtc) {
#pragma unroll
        for (int v = 0; v < 16; ++v) ST[mtc][v] = st[(r_own + ln) * C::D + 32 * mtc + acc_row(v, h)];
    }
    macc = (h == 0) ? st[C::LR * C::D + r_own + ln] : 0.f;

    const int64_t t_begin = seg * a.seg_len;
    const int64_t t_end = (t_begin + a.seg_len < a.N) ? t_begin + a.seg_len : a.N;
    const int ntiles = static_cast<int>((t_end - t_begin + kTile - 1) / kTile);
    auto tile_t0 = [&](int it) { return t_begin + static_cast<int64_t>(kReverse ? ntiles - 1 - it : it) * kTile; };
    auto tile_nv = [&](int64_t t0) { return (t_end - t0 < kTile) ? static_cast<int>(t_end - t0) : kTile; };

    // loads run ahead of the arithmetic: issued when few registers are live, written to LDS at the next tile's start
    RowChunks<C, kTile> pre_r, pre_w, pre_v;
    CotChunks<C, kTile> pre_c;
    auto fetch = [&](int it) {
        const int64_t t0 = tile_t0(it);
        const int nv = tile_nv(t0);
        fetch_rows<C, kTile>(Xr, t0, nv, pre_r);
        if (intra) fetch_rows<C, kTile>(Xw, t0, nv, pre_w);
        if (SIDE == 1 || intra) fetch_rows<C, kTile>(V, t0, nv, pre_v);
        if (SIDE == 0 || intra) fetch_cotangent<C, kTile>(dO, O, den, t0, nv, pre_c);
    };
    if (ntiles > 0) fetch(0);

    GRAD_PHASE_DECL
    for (int it = 0; it < ntiles; ++it) {
        const int64_t t0 = tile_t0(it);
        const int nvalid = tile_nv(t0);

        // ---- registers -> LDS
        store_rows<C, kTile>(pre_r, xr);
        if (intra) store_rows<C, kTile>(pre_w, xw);
        if (SIDE == 0) {
            store_cotangent<C, kTile>(pre_c, yr, sr);
            if (intra) store_rows<C, kTile>(pre_v, yw);
            if (tid < kTile) sw[tid] = 1.f;
        } else {
            store_rows<C, kTile>(pre_v, yr);
            if (intra) store_cotangent<C, kTile>(pre_c, yw, sw);
            if (tid < kTile) sr[tid] = 1.f;
        }
        GRAD_PHASE(0)
        __syncthreads();
        GRAD_PHASE(1)

        // extra columns as bf16 (hi, lo) pairs: three products hi*hi + hi*lo + lo*hi keep 16 mantissa bits
        float sr_hi, sr_lo;
        split_bf16(sr[ln], sr_hi, sr_lo);
        const u32x4 sr_a = (h == 0) ? u32x4{pack2(sr_hi, sr_hi), pack2(sr_lo, 0.f), 0u, 0u} : u32x4{0u, 0u, 0u, 0u};

        // ---- production, by role: the first NGW*TPL wavefronts hash the writer's tables; the last NGW
        //      project the reader (kept for the backward pass through the soft assignment); one more forms
        //      the in-tile term T^T[b][a] = Yw_b . Yr_a + sw_b * sr_a, masked, as MFMA operands for everybody
        if (intra && w < G::NGW * C::TPL) {
            const int pg = w % G::NGW, pj = w / G::NGW;
            const f32x16 zw = project<C>(wp, xw, th * G::NGW + pg, ln, h);
            write_assignments<C>(zw, th * G::NGW + pg, ln, h, a.beta, ln < nvalid, phw, pj, C::TPL);
        }
        if (w >= kWaves - G::NGW) {
            const int pg = kWaves - 1 - w;
            const f32x16 zr = project<C>(wp, xr, th * G::NGW + pg, ln, h);
            float *zdst = zl + (pg * 64 + lane) * 16;
#pragma unroll
            for (int v = 0; v < 16; v += 4) *reinterpret_cast<float4 *>(zdst + v) = float4{zr[v], zr[v + 1], zr[v + 2], zr[v + 3]};
        }
        if (intra && w == kWaves - 1 - G::NGW) {
            f32x16 tt = {0};
            const int yo = opaque(ln * C::XS + 8 * h);
#pragma unroll
            for (int s = 0; s < C::D / 16; ++s) tt = mma(lds128(yw + yo + 16 * s), lds128(yr + yo + 16 * s), tt);
            float sw_hi, sw_lo;
            split_bf16(sw[ln], sw_hi, sw_lo);
            const u32x4 sw_a = (h == 0) ? u32x4{pack2(sw_hi, sw_hi), pack2(sw_lo, 0.f), 0u, 0u} : u32x4{0u, 0u, 0u, 0u};
            const u32x4 sr_b = (h == 0) ? u32x4{pack2(sr_hi, sr_lo), pack2(sr_hi, 0.f), 0u, 0u} : u32x4{0u, 0u, 0u, 0u};
            tt = mma(sw_a, sr_b, tt);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int b = acc_row(v, h);
                const bool keep = kReverse ? (b >= ln) : (b <= ln);
                tt[v] = keep ? tt[v] : 0.f;
            }
            ttop[lane] = acc_operand(tt, 0);
            ttop[64 + lane] = acc_operand(tt, 1);
        }
        GRAD_PHASE(2)
        __syncthreads();
        GRAD_PHASE(3)
        GRAD_PHASE(4)
        // ---- cotangent of the reader's assignments for this wavefront's 32 bucket rows
        f32x16 dP;
        {
            // extra column first: sr_a * (A or dA)[r] with the masses before this tile
            float m_hi, m_lo;
            split_bf16(macc + __shfl_xor(macc, 32, 64), m_hi, m_lo);
            const u32x4 mb = (h == 0) ? u32x4{pack2(m_hi, m_lo), pack2(m_hi, 0.f), 0u, 0u} : u32x4{0u, 0u, 0u, 0u};
            dP = mma(sr_a, mb, f32x16{0});
        }
        if (intra) {
#pragma unroll
            for (int s = 0; s < 2; ++s)
                dP = mma(ttop[64 * s + lane], lds_tr_acc(phw, C::PS, 16 * s, r_own, ln, h), dP);
        }
        {
            const int yo = opaque(ln * C::XS + 4 * h);
#pragma unroll
            for (int mtc = 0; mtc < C::NT; ++mtc) {
#pragma unroll
                for (int s = 0; s < 2; ++s) {
                    const int cc = 32 * mtc + 16 * s;
                    dP = mma(lds64x2(yr + yo + cc, yr + yo + cc + 8), acc_operand(ST[mtc], s), dP);
                }
            }
        }
        GRAD_PHASE(5)
        // ---- statistics += Yw^T . phi_writer
        if (intra) {
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const float4 g0 = *reinterpret_cast<const float4 *>(sw + 16 * s + 8 * h);
                const float4 g1 = *reinterpret_cast<const float4 *>(sw + 16 * s + 8 * h + 4);
                const u32x4 bp = lds_tr_plain(phw, C::PS, 16 * s, r_own, ln, h);
                macc += bf_lo(bp.x) * g0.x + bf_hi(bp.x) * g0.y + bf_lo(bp.y) * g0.z + bf_hi(bp.y) * g0.w +
                        bf_lo(bp.z) * g1.x + bf_hi(bp.z) * g1.y + bf_lo(bp.w) * g1.z + bf_hi(bp.w) * g1.w;
#pragma unroll
                for (int mtc = 0; mtc < C::NT; ++mtc)
                    ST[mtc] = mma(lds_tr_plain(yw, C::XS, 16 * s, 32 * mtc, ln, h), bp, ST[mtc]);
            }
        }
        GRAD_PHASE(6)
        __syncthreads();        // phase-A tiles are dead from here on
        GRAD_PHASE(7)

        // ---- hand the cotangents to the lanes that own (token, table)
        {
            const int dbase = opaque(4 * h * S::DS + (r_own - r_base) + ln);
#pragma unroll
            for (int v = 0; v < 16; ++v) dphi[dbase + (8 * (v >> 2) + (v & 3)) * S::DS] = dP[v];
        }
        // the next tile's loads fly during the vector-ALU phases below (few registers are live here)
        if (it + 1 < ntiles) fetch(it + 1);
        GRAD_PHASE(8)
        __syncthreads();
        GRAD_PHASE(9)

        // ---- back through the corner softmax and tanh (Algorithm 1, step 4):
        //      with w_r = phi_r dphi_r, m = sum_r w_r, E_t = sum_r v_{r,t} w_r:
        //      du_t = beta (E_t - m (p_t - q_t)),  dz_t = du_t (1 - tanh^2 z_t)
        //      The R corners of a table are split over AW wavefronts by their high bits; wavefronts aq > 0
        //      hand their partial sums (m, E_t) to wavefront aq == 0 of the same table through LDS.
        float Efin[C::P + 1];          // aq == 0 only: E_t and m after combining (last table of the lane)
        float p_k[C::P], q_k[C::P], s_k[C::P];
        int jfin = -1;
#pragma unroll
        for (int j = 0; j < C::TPL; ++j) {
            const int table = g * C::TPG + h * C::TPL + j;
            if (table >= C::L) break;
            if (j < jq || (j - jq) % G::JW != 0) continue;
            constexpr int ZW = C::PP;                              // the table's slots are contiguous
            f32x16 z = {0};
            {
                const float *zsrc = zl + (gl * 64 + lane) * 16 + ZW * j;
#pragma unroll
                for (int v = 0; v < ZW; v += 4) {
                    const float4 z4 = *reinterpret_cast<const float4 *>(zsrc + v);
                    z[ZW * j + v] = z4.x; z[ZW * j + v + 1] = z4.y; z[ZW * j + v + 2] = z4.z; z[ZW * j + v + 3] = z4.w;
                }
            }
            float p[C::P], q[C::P], sech2[C::P], lo[1 << C::PLO], hi[1 << C::PHI];
            bit_masses<C>(z, j, a.beta, p, q, sech2);
            kron_factors<C>(p, q, lo, hi);
            const int dsrc = opaque(ln * S::DS + (table * C::R - r_base));
            float E[C::P];
#pragma unroll
            for (int t = 0; t < C::P; ++t) E[t] = 0.f;
            float m = 0.f;
#pragma unroll
            for (int aa = 0; aa < (1 << C::PHI); ++aa) {
                if (aa < a0 || aa >= a0 + G::AN) continue;
                const float *src = dphi + dsrc + aa * 8;
                const float4 d0 = *reinterpret_cast<const float4 *>(src);
                const float4 d1 = *reinterpret_cast<const float4 *>(src + 4);
                const float wv[8] = {hi[aa] * lo[0] * d0.x, hi[aa] * lo[1] * d0.y, hi[aa] * lo[2] * d0.z, hi[aa] * lo[3] * d0.w,
                                     hi[aa] * lo[4] * d1.x, hi[aa] * lo[5] * d1.y, hi[aa] * lo[6] * d1.z, hi[aa] * lo[7] * d1.w};
                const float s01 = wv[0] + wv[1], s23 = wv[2] + wv[3], s45 = wv[4] + wv[5], s67 = wv[6] + wv[7];
                E[0] += ((wv[1] - wv[0]) + (wv[3] - wv[2])) + ((wv[5] - wv[4]) + (wv[7] - wv[6]));
                if (C::PLO > 1) E[1] += (s23 - s01) + (s67 - s45);
                const float s0123 = s01 + s23, s4567 = s45 + s67;
                if (C::PLO > 2) E[2] += s4567 - s0123;
                const float chunk = s0123 + s4567;
                m += chunk;
#pragma unroll
                for (int t = 0; t < C::PHI; ++t) E[C::PLO + t] += ((aa >> t) & 1) ? chunk : -chunk;
                RACE_SCHED_FENCE();
            }
            if (G::AW > 1 && aq > 0) {
                float *dst = part + (((aq - 1) * G::NGW * G::JW + (w % (G::NGW * G::JW))) * 64 + lane) * 8;
                *reinterpret_cast<float4 *>(dst) = float4{m, E[0], E[1], E[2]};
                *reinterpret_cast<float4 *>(dst + 4) = float4{C::P > 3 ? E[3 % C::P] : 0.f, C::P > 4 ? E[4 % C::P] : 0.f,
                                                              C::P > 5 ? E[5 % C::P] : 0.f, C::P > 6 ? E[6 % C::P] : 0.f};
            }
            if (G::AW == 1) {
                // one wavefront sees the whole table: finish here
                float dzv[ZW];
#pragma unroll
                for (int t = 0; t < ZW; ++t) dzv[t] = (t < C::P) ? a.beta * (E[t] - m * (p[t] - q[t])) * sech2[t] : 0.f;
#pragma unroll
                for (int t = 0; t < ZW; t += 4) {
                    const int v = ZW * j + t;      // slot v of the projection accumulator is projection row acc_row(v, h)
                    *reinterpret_cast<u32x2 *>(dz + ln * S::DZS + gl * 32 + 8 * (v >> 2) + 4 * h) =
                        u32x2{pack2(dzv[t], dzv[t + 1]), pack2(dzv[t + 2], dzv[t + 3])};
                }
            } else {
                jfin = j;
                Efin[C::P] = m;
#pragma unroll
                for (int t = 0; t < C::P; ++t) { Efin[t] = E[t]; p_k[t] = p[t]; q_k[t] = q[t]; s_k[t] = sech2[t]; }
            }
        }
        if (G::AW > 1) {
            __syncthreads();
            if (aq == 0 && jfin >= 0) {
#pragma unroll
                for (int o = 1; o < G::AW; ++o) {
                    const float *src = part + (((o - 1) * G::NGW * G::JW + (w % (G::NGW * G::JW))) * 64 + lane) * 8;
                    const float4 p0 = *reinterpret_cast<const float4 *>(src);
                    const float4 p1 = *reinterpret_cast<const float4 *>(src + 4);
                    const float pe[8] = {p0.x, p0.y, p0.z, p0.w, p1.x, p1.y, p1.z, p1.w};
                    Efin[C::P] += pe[0];
#pragma unroll
                    for (int t = 0; t < C::P; ++t) Efin[t] += pe[1 + t];
                }
                constexpr int ZW = C::PP;
                float dzv[ZW];
#pragma unroll
                for (int t = 0; t < ZW; ++t)
                    dzv[t] = (t < C::P) ? a.beta * (Efin[t % C::P] - Efin[C::P] * (p_k[t % C::P] - q_k[t % C::P])) * s_k[t % C::P] : 0.f;
#pragma unroll
                for (int t = 0; t < ZW; t += 4) {
                    const int v = ZW * jfin + t;
                    *reinterpret_cast<u32x2 *>(dz + ln * S::DZS + gl * 32 + 8 * (v >> 2) + 4 * h) =
                        u32x2{pack2(dzv[t], dzv[t + 1]), pack2(dzv[t + 2], dzv[t + 3])};
                }
            }
        }
        GRAD_PHASE(10)
        __syncthreads();
        GRAD_PHASE(11)

        // ---- this workgroup's columns of dZ (projection rows of its groups) -> workspace, 16-byte pieces
        if (tid < kTile * G::NGW * 4) {
            const int row = tid / (G::NGW * 4), ch = tid % (G::NGW * 4);
            if (row < nvalid)
                *reinterpret_cast<u32x4 *>(dZ + (t0 + row) * C::LPP + th * G::NGW * 32 + 8 * ch) =
                    *reinterpret_cast<const u32x4 *>(dz + row * S::DZS + 8 * ch);
        }
        GRAD_PHASE(12)
        __syncthreads();
        GRAD_PHASE(1)
    }
    GRAD_PHASE_PRINT()
}

// dX = dZ . W: (N x LPP) . (LPP x d) per head; a workgroup of NT wavefronts takes kDzTiles tiles of 32 tokens.
constexpr int kDzTiles = 8;
template <class C>
__global__ __launch_bounds__(64 * C::NT)
void dz_matmul_kernel(KArgs a, const bf16raw *dZ, bf16raw *dX)
{
    constexpr int SS = 40;
    __shared__ __attribute__((aligned(16))) bf16raw dz[kTile * C::ZS];
    __shared__ __attribute__((aligned(16))) bf16raw stage[C::NT * kTile * SS];
    const int bh = blockIdx.y, head = bh % a.H;
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, ln = lane & 31, h = lane >> 5;
    dZ += static_cast<size_t>(bh) * a.N * C::LPP;
    dX += static_cast<size_t>(bh) * a.N * C::D;
    const bf16raw *wt = a.WpT + static_cast<size_t>(head) * C::D * C::LPP;     // [d][LPP]
    const int nt = w;
    u32x4 bw[C::LPP / 16];
#pragma unroll
    for (int s = 0; s < C::LPP / 16; ++s)
        bw[s] = *reinterpret_cast<const u32x4 *>(wt + (32 * nt + ln) * C::LPP + 16 * s + 8 * h);
    for (int k = 0; k < kDzTiles; ++k) {
        const int64_t t0 = (static_cast<int64_t>(blockIdx.x) * kDzTiles + k) * kTile;
        if (t0 >= a.N) break;
        const int nvalid = (a.N - t0 < kTile) ? static_cast<int>(a.N - t0) : kTile;
        __syncthreads();
        for (int c = tid; c < kTile * (C::LPP / 8); c += 64 * C::NT) {
            const int row = c / (C::LPP / 8), ch = c % (C::LPP / 8);
            u32x4 v = {0, 0, 0, 0};
            if (row < nvalid) v = *reinterpret_cast<const u32x4 *>(dZ + (t0 + row) * C::LPP + 8 * ch);
            *reinterpret_cast<u32x4 *>(dz + row * C::ZS + 8 * ch) = v;
        }
        __syncthreads();
        f32x16 acc = {0};
#pragma unroll
        for (int s = 0; s < C::LPP / 16; ++s) acc = mma(lds128(dz + ln * C::ZS + 16 * s + 8 * h), bw[s], acc);
        bf16raw *sg = stage + w * kTile * SS;
#pragma unroll
        for (int v = 0; v < 16; ++v) sg[acc_row(v, h) * SS + ln] = static_cast<bf16raw>(pack2(acc[v], 0.f) & 0xffffu);
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            const int row = (lane >> 2) + 16 * kk, ch = lane & 3;
            const u32x4 piece = *reinterpret_cast<const u32x4 *>(sg + row * SS + 8 * ch);
            if (row < nvalid) *reinterpret_cast<u32x4 *>(dX + (t0 + row) * C::D + 32 * nt + 8 * ch) = piece;
        }
    }
}

}  // namespace mfma
}  // namespace race
