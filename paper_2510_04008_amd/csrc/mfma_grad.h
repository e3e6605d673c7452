// grad_kernel: the two backward passes that contract the bucket statistics over the head dimension.
// Register budget: with eight wavefronts of 256 registers a wavefront can carry up to 64 bucket rows x 128
// columns of fp32 statistics (128 registers) next to its working set, i.e. 512 bucket rows per workgroup.
// The workgroup then also forms dX = dz . W for its tile.  (Shapes with more bucket rows than that are not compiled.)
//
//   SIDE 0 (dQ), left to right, statistics S = (B | A) of (phi_K, [V | 1]) before/with token i:
//       dphi_Q(i)[r] = S[r,:] . [dO_i/e_i | -(dO_i.O_i)/e_i]
//   SIDE 1 (dK), right to left, statistics dS = (dB | dA) of (phi_Q, read-out cotangents) of tokens >= j:
//       dphi_K(j)[r] = dS[r,:] . [V_j | 1]
// followed in both cases by the chain rule through the corner softmax, tanh and W:  dx = W^T dz.
// "reader" is the tensor whose gradient is produced, "writer" the tensor that feeds the statistics.  The writer's
// assignments are rebuilt from its hashed rows (hash_kernel); the reader's rows are projected here, because the chain
// rule needs tanh and its derivative next to the per-bit masses.
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

// Row tiles per wavefront: all of LR / 256 if that is at most two (128 registers of statistics per lane is what
// fits next to the working set); beyond that the bucket rows are split over TSPLIT workgroups by tables.
template <class C> constexpr int grad_row_tiles() { return C::LR / (32 * kWaves) >= 2 ? 2 : 1; }

template <class C>
struct GradCfg {
    static constexpr int MTG = grad_row_tiles<C>();                     // 32-row tiles of bucket rows per wavefront
    static constexpr int RW = 32 * MTG;                                 // bucket rows per wavefront
    static constexpr int NRW = C::LR / RW >= kWaves ? kWaves : C::LR / RW;   // wavefronts that own bucket rows (the first NRW)
    static constexpr int TSPLIT = C::LR / (RW * NRW);                   // workgroups per (segment, head)
    static constexpr int NGW = C::NG / TSPLIT;                          // projection groups per workgroup
    static constexpr int ROWS = C::LR / TSPLIT;                         // bucket rows per workgroup
    static constexpr int TABLES = NGW * C::TPG;                         // tables per workgroup
    // a wavefront's rows are TWW whole tables (R <= RW) or a 1/WPT share of one table (R > RW);
    // a 32-row tile holds TW whole tables (R <= 32) or part of one
    static constexpr int TWW = C::R >= RW ? 1 : RW / C::R;              // tables per wavefront
    static constexpr int WPT = C::R >= RW ? C::R / RW : 1;              // wavefronts per table
    static constexpr int TW = C::R >= 32 ? 1 : 32 / C::R;               // tables per tile
    static constexpr int KM = (C::R >= 32 ? 32 : C::R) / 8;             // groups of 8 corners per table and tile
    static constexpr int MB = KM == 4 ? 2 : (KM == 2 ? 1 : 0);          // corner bits 3.. that vary inside a tile
    static_assert(MTG >= 1 && NRW >= 1 && TSPLIT == 1 && RW * NRW == C::LR, "all bucket rows of a head in one workgroup");
    static_assert(NRW == kWaves || TSPLIT == 1, "a workgroup with spare wavefronts holds all the rows");
    static_assert(C::NG % TSPLIT == 0 && kWaves % NGW == 0, "table split");
    static_assert(NGW * C::TPG * C::R >= ROWS, "a workgroup's rows are the tables of its projection groups");
    static_assert(C::P >= 3 && C::P <= 7, "corner bits 0..2 are register/lane bits; a partial record is P+1 <= 8 floats");
    // production roles.  Writer hashing: one wavefront per (projection group, table of the lane, share of the
    // high-bit indices); reader masses: one per (projection group, table of the lane) if there is room, else one
    // per projection group; one wavefront for the in-tile term.  If they do not all fit, the reader and in-tile
    // roles double up on the last wavefronts.
    static constexpr int AS = (C::PHI >= 2 && NGW * C::TPL * 2 + NGW + 1 <= kWaves) ? 2 : 1;     // shares hold pairs of indices
    static constexpr int NW = NGW * C::TPL * AS;                        // writer wavefronts
    // (where every wavefront carries statistics, a wavefront is kept free for the in-tile term; where some do not,
    // it doubles up on a reader: measured faster each way)
    static constexpr int RJ = (NW + NGW * C::TPL + (NRW < kWaves ? 0 : 1) <= kWaves) ? C::TPL : 1;
    static constexpr bool DISJ = NW + NGW * RJ + 1 <= kWaves;
    static constexpr int RD0 = DISJ ? NW : kWaves - NGW * RJ;           // first reader wavefront
    static constexpr int NR = NGW * RJ;                                 // reader wavefronts
    // in-tile term: a wavefront of its own if one is left, else the last reader
    static constexpr int TT = DISJ ? (NW + NR < kWaves ? NW + NR : kWaves - 1) : kWaves - 1 - NGW;
    static_assert(NW <= kWaves && RD0 + NR <= kWaves, "production roles must fit the wavefronts");
    // dX = dz . W of a tile is formed one step late, next to the production of the following tile, by the wavefronts
    // with the lightest production roles: first those without a role, then the in-tile term's, then writers,
    // readers last (the higher wavefront first within a class).  dx_tile(w) = column tile of wavefront w, or -1.
    // The non-causal variant has no writer and no in-tile term: its readers start at wavefront 0 and take one table of
    // the lane each if the wavefronts suffice.
    static constexpr int RJ_NC = NGW * C::TPL <= kWaves ? C::TPL : 1;
    static constexpr int NR_NC = NGW * RJ_NC;
    static constexpr int role_weight(int w, bool causal)
    {
        if (!causal) return w < NR_NC ? 3 : 0;
        return (w >= RD0 && w < RD0 + NR) ? 3 : (w < NW ? 2 : (w == TT ? 1 : 0));
    }
    static constexpr int dx_tile(int w, bool causal)
    {
        int taken = 0;
        for (int weight = 0; weight <= 3; ++weight) {
            for (int v = kWaves - 1; v >= 0; --v) {
                if (role_weight(v, causal) != weight) continue;
                if (taken == C::NT) return -1;
                if (v == w) return taken;
                ++taken;
            }
        }
        return -1;
    }
};

// UNIT: the unit-norm option's extras (row scales, parts of z . dz, and z next to the per-bit masses).
// INTRA: the causal variant, whose tiles also feed the statistics: the writer's rows, assignments and the in-tile term.
template <class C, bool UNIT, bool INTRA>
struct GradLds {
    using G = GradCfg<C>;
    static constexpr int wp = 0;                                        // [LPP][XS] bf16
    static constexpr int DZS = G::NGW * 32 + 8;                         // bf16 row stride of the dz tile
    static constexpr int dz = wp + C::LPP * C::XS * 2;                  // [32][DZS] bf16
    static constexpr int sr = dz + kTile * DZS * 2;                     // [32] fp32 extra column of reader-Y
    static constexpr int sw = sr + kTile * 4;                           // [32] fp32 extra column of writer-Y
    static constexpr int nrm = sw + kTile * 4;                          // [2][2][32] fp32: 1 / |x| of the reader and writer rows (unit-norm option),
                                                                        // two buffers used by alternate tiles
    static constexpr int rad = nrm + (UNIT ? 4 * kTile * 4 : 0);        // [kWaves][32] fp32: per-wavefront parts of z . dz per token (same option)
    static constexpr int PMS = UNIT ? 5 * C::PP + (C::PP == 8 ? 4 : 8)  // floats per (table, token): p, q, sech^2, tanh (, z), each padded
                                    : 4 * C::PP + 4;                    // to PP; the tail makes PMS / 4 odd, which keeps 16-byte reads of
                                                                        // 16 tokens on distinct banks
    static constexpr int pm = (rad + (UNIT ? kWaves * kTile * 4 : 0) + 15) & ~15;              // [TABLES][32][PMS] fp32: per-bit masses of the reader
    static constexpr int PMT = G::TABLES < C::L ? G::TABLES : C::L;     // tables of the workgroup that exist
    static constexpr int part = pm + PMT * kTile * PMS * 4;             // [kWaves][32][8] fp32: partial (m, G_t) of table shares
    static constexpr int yr = part + (G::WPT > 1 ? kWaves * kTile * 8 * 4 : 0);   // [32][XS] reader-Y rows, pair-interleaved columns
    static constexpr int ttop = yr + kTile * C::XS * 2;                 // [2][64] x 16 B: masked in-tile term as MFMA operands
    static constexpr int xr = (ttop + (INTRA ? 2 * 64 * 16 : 0) + 255) & ~255;        // [32][XS]
    static constexpr int mw = xr + kTile * C::XS * 2;                   // [32][MS] fp32: hashed writer rows
    static constexpr int yw = (mw + (INTRA ? kTile * C::MS * 4 : 0) + 15) & ~15;     // [32][YS] writer-Y rows, pair-interleaved columns
    static constexpr int phw = yw + (INTRA ? kTile * C::YS * 2 : 0);    // [32][PST] writer assignments
    static constexpr int SS = 40;                                       // bf16 row stride of the output staging tiles
    static constexpr int stg = phw + (INTRA ? kTile * C::PST * 2 : 0);  // [NT][32][SS] bf16: dX tiles on their way out
    static constexpr int xr2 = stg + C::NT * kTile * SS * 2;            // [32][XS]: second buffer of the reader rows (unit-norm
                                                                        // option: the dX wavefronts still read a tile's rows while the others
                                                                        // store the next tile's)
    static constexpr int total = xr2 + (UNIT ? kTile * C::XS * 2 : 0);
    static_assert(total <= 160 * 1024, "LDS budget");
};

// Wavefronts per SIMD the gradient kernel is compiled for.  The non-causal variant of a shape whose wavefronts carry
// at most two accumulator tiles of statistics fits 128 registers and 80 KB of LDS, which lets two workgroups share a CU
// (its tiles are independent of each other: nothing but latency to hide).
template <class C, bool UNIT, bool INTRA>
constexpr int grad_waves_per_simd()
{
    return (!INTRA && GradCfg<C>::MTG * C::NT <= 2 && GradLds<C, UNIT, INTRA>::total <= 80 * 1024) ? 4 : 2;
}

template <class C, int SIDE, bool UNIT, bool INTRA>
__global__ __launch_bounds__(kThreads, (grad_waves_per_simd<C, UNIT, INTRA>()))
void grad_kernel(KArgs a, const bf16raw *Q, const bf16raw *K, const bf16raw *V, const bf16raw *O,
                 const float *den, const bf16raw *dO, bf16raw *dX)
{
    using S = GradLds<C, UNIT, INTRA>;
    using G = GradCfg<C>;
    extern __shared__ __attribute__((aligned(256))) unsigned char lds[];
    bf16raw *wp = reinterpret_cast<bf16raw *>(lds + S::wp);
    bf16raw *dz = reinterpret_cast<bf16raw *>(lds + S::dz);
    float *sr = reinterpret_cast<float *>(lds + S::sr);
    float *sw = reinterpret_cast<float *>(lds + S::sw);
    float *nrm0 = reinterpret_cast<float *>(lds + S::nrm);
    float *rad = reinterpret_cast<float *>(lds + S::rad);
    float *pm = reinterpret_cast<float *>(lds + S::pm);
    bf16raw *yr = reinterpret_cast<bf16raw *>(lds + S::yr);
    bf16raw *xr0 = reinterpret_cast<bf16raw *>(lds + S::xr);
    float *mw = reinterpret_cast<float *>(lds + S::mw);
    bf16raw *yw = reinterpret_cast<bf16raw *>(lds + S::yw);
    bf16raw *phw = reinterpret_cast<bf16raw *>(lds + S::phw);
    float *part = reinterpret_cast<float *>(lds + S::part);
    u32x4 *ttop = reinterpret_cast<u32x4 *>(lds + S::ttop);
    bf16raw *stg = reinterpret_cast<bf16raw *>(lds + S::stg);

    constexpr bool kReverse = (SIDE == 1);
    const int seg = blockIdx.x, bh = blockIdx.y, head = bh % a.H;
    const int tid = threadIdx.x, w = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, ln = lane & 31, h = lane >> 5;
    constexpr int th = 0;                            // (a workgroup owns all the tables)
    const int r_base = th * G::ROWS;                 // its first bucket row
    const int r_own = r_base + w * G::RW;            // this wavefront's bucket rows
    // backward pass through the soft assignment: the tables (or the share of one table) behind this wavefront's rows
    const int tl0 = (w * G::RW) / C::R;              // first table, counted inside the workgroup
    const int ro = (w * G::RW) % C::R;               // first corner of the share (0 unless a table spans several wavefronts)
    constexpr bool intra = INTRA;
    // shapes with fewer than 8 x 32 bucket rows: only the first NRW wavefronts carry statistics; the others take
    // part in the production, the loads and dX
    const bool has_rows = G::NRW == kWaves || w < G::NRW;

    const size_t base = static_cast<size_t>(bh) * a.N * C::D;
    Q += base; K += base; V += base; O += base; dO += base;
    dX += base;
    den += static_cast<size_t>(bh) * a.N;
    const bf16raw *Xr = SIDE == 0 ? Q : K;
    const float *Mw = (SIDE == 0 ? a.Mk : a.Mq) + static_cast<size_t>(bh) * a.N * C::LP;
    const float *st = a.state + (static_cast<size_t>(bh) * a.nseg + seg) * C::STATE;

    {
        const bf16raw *src = a.Wp + static_cast<size_t>(head) * C::LPP * C::D;
        for (int c = tid; c < C::LPP * C::CPR; c += kThreads) {
            const int row = c / C::CPR, ch = c % C::CPR;
            *reinterpret_cast<u32x4 *>(wp + row * C::XS + ch * 8) = *reinterpret_cast<const u32x4 *>(src + row * C::D + ch * 8);
        }
    }
    if (G::TABLES * C::R != G::ROWS || C::TPG * C::PP < 32) {
        // projection slots of tables that do not exist are never written below: they must be zeros for dX = dz . W
        for (int i = tid; i < kTile * S::DZS; i += kThreads) dz[i] = 0;
    }
    // statistics at the start of the segment, transposed tiles ST[row tile][column tile]: columns x 32 bucket rows
    f32x16 ST[G::MTG][C::NT];
    float macc[G::MTG];       // extra column (A or dA): per-half partial sum, lane n <-> row r_own + 32 mr + n
#pragma unroll
    for (int mr = 0; mr < G::MTG; ++mr) {
#pragma unroll
        for (int mtc = 0; mtc < C::NT; ++mtc) {
#pragma unroll
            for (int v = 0; v < 16; ++v)
                ST[mr][mtc][v] = has_rows ? st[(r_own + 32 * mr + ln) * C::D + 32 * mtc + acc_row(v, h)] : 0.f;
        }
        macc[mr] = (has_rows && h == 0) ? st[C::LR * C::D + r_own + 32 * mr + ln] : 0.f;
    }

    const int64_t t_begin = seg * a.seg_len;
    const int64_t t_end = (t_begin + a.seg_len < a.N) ? t_begin + a.seg_len : a.N;
    const int ntiles = static_cast<int>((t_end - t_begin + kTile - 1) / kTile);
    auto tile_t0 = [&](int it) { return t_begin + static_cast<int64_t>(kReverse ? ntiles - 1 - it : it) * kTile; };
    auto tile_nv = [&](int64_t t0) { return (t_end - t0 < kTile) ? static_cast<int>(t_end - t0) : kTile; };

    // loads run ahead of the arithmetic: issued a step ahead, written to LDS at the next tile's start
    RowChunks<C, kTile> pre_r, pre_v;
    MassChunks<C, kTile> pre_w;
    CotChunks<C, kTile> pre_c;
    auto fetch = [&](int it) {
        const int64_t t0 = tile_t0(it);
        const int nv = tile_nv(t0);
        fetch_rows<C, kTile, true>(Xr, t0, nv, pre_r);
        if (intra) fetch_masses<C, kTile>(Mw, t0, nv, pre_w);
        if (SIDE == 1 || intra) fetch_rows<C, kTile, true>(V, t0, nv, pre_v);
        if (SIDE == 0 || intra) fetch_cotangent<C, kTile, true>(dO, O, den, t0, nv, pre_c);
    };
    if (ntiles > 0) fetch(0);

    // ---- dX = dz . W for one tile (the chain rule through W): a wavefront forms the transposed 32 x 32 tile of its
    //      column tile nt (lane = token, registers = columns 32 nt + acc_row(v, h)), stages it in its own corner of
    //      LDS and stores 16-byte row pieces; nobody else touches that corner.  Called one step late (after the
    //      next tile's first barrier, which also publishes dz), so that it runs next to the production phase
    //      instead of keeping everybody waiting at the end of the tile; xr_t, nrm_t: the tile's reader rows and scales
    //      (unit-norm option).
    static_assert(C::NT <= kWaves, "one wavefront per column tile");
    auto dx_stage = [&](int nt, int64_t t0, int nvalid, const bf16raw *xr_t, const float *nrm_t) __attribute__((always_inline)) {
        const int lo = opaque(lane);                     // addresses below are rebuilt per tile, not kept in registers
        const int lno = lo & 31, ho = lo >> 5;
        f32x16 acc = {0};
#pragma unroll
        for (int s = 0; s < C::LPP / 16; ++s)
            acc = mma(lds_tr_plain(wp, C::XS, 16 * s, 32 * nt, lno, ho), lds128(dz + lno * S::DZS + 16 * s + 8 * ho), acc);
        if (UNIT) {
            float cp = 0.f;                              // (z . dz) / |x|^2 of token lno, parts in wavefront order
#pragma unroll
            for (int i = 0; i < kWaves; ++i) cp += rad[i * kTile + lno];
            cp *= nrm_t[lno];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const u32x2 xv = *reinterpret_cast<const u32x2 *>(xr_t + lno * C::XS + 32 * nt + 8 * k + 4 * ho);
                acc[4 * k] = fmaf(-cp, bf_lo(xv.x), acc[4 * k]);
                acc[4 * k + 1] = fmaf(-cp, bf_hi(xv.x), acc[4 * k + 1]);
                acc[4 * k + 2] = fmaf(-cp, bf_lo(xv.y), acc[4 * k + 2]);
                acc[4 * k + 3] = fmaf(-cp, bf_hi(xv.y), acc[4 * k + 3]);
            }
        }
        bf16raw *sg = stg + nt * kTile * S::SS;
#pragma unroll
        for (int k = 0; k < 4; ++k)
            *reinterpret_cast<u32x2 *>(sg + lno * S::SS + 8 * k + 4 * ho) =
                u32x2{pack2(acc[4 * k], acc[4 * k + 1]), pack2(acc[4 * k + 2], acc[4 * k + 3])};
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            const int row = (lo >> 2) + 16 * kk, ch = lo & 3;
            const u32x4 piece = *reinterpret_cast<const u32x4 *>(sg + row * S::SS + 8 * ch);
            if (row < nvalid) *reinterpret_cast<u32x4 *>(dX + (t0 + row) * C::D + 32 * nt + 8 * ch) = piece;
        }
    };
    // this wavefront's column tile of dX (-1: none), by table look-up over the compile-time assignment
    int my_dx = -1;
#pragma unroll
    for (int v = 0; v < kWaves; ++v)
        if (w == v) my_dx = G::dx_tile(v, INTRA);
    auto tile_xr = [&](int it) { return (UNIT && (it & 1)) ? reinterpret_cast<bf16raw *>(lds + S::xr2) : xr0; };
    auto tile_nrm = [&](int it) { return nrm0 + ((UNIT && (it & 1)) ? 2 * kTile : 0); };

    float dbeta_acc = 0.f;    // this lane's share of the cotangent of beta: sum of (E_t - m (p_t - q_t)) tanh z_t
    GRAD_PHASE_DECL
    for (int it = 0; it < ntiles; ++it) {
        const int64_t t0 = tile_t0(it);
        const int nvalid = tile_nv(t0);
        // unit-norm option: alternate tiles use alternate buffers for the reader's rows and the scales
        bf16raw *xr = tile_xr(it);
        float *nrm = tile_nrm(it);

        // ---- registers -> LDS
        store_rows<C, kTile>(pre_r, xr, nvalid);
        if (intra) store_masses<C, kTile>(pre_w, mw);
        if (UNIT) store_row_scales<C, kTile>(pre_r, nrm);
        if (SIDE == 0) {
            store_cotangent<C, kTile, C::XS, true>(pre_c, yr, sr, a.L_real, nvalid);
            if (intra) store_rows<C, kTile, C::YS, true>(pre_v, yw, nvalid);
            if (tid < kTile) sw[tid] = 1.f;
        } else {
            store_rows<C, kTile, C::XS, true>(pre_v, yr, nvalid);
            if (intra) store_cotangent<C, kTile, C::YS, true>(pre_c, yw, sw, a.L_real, nvalid);
            if (tid < kTile) sr[tid] = 1.f;
        }
        GRAD_PHASE(0)
        __syncthreads();
        GRAD_PHASE(1)
        if (it > 0 && my_dx >= 0) {
            const int64_t tp = tile_t0(it - 1);
            dx_stage(my_dx, tp, tile_nv(tp), tile_xr(it - 1), tile_nrm(it - 1));
        }
        GRAD_PHASE(12)

        // extra columns as bf16 (hi, lo) pairs: three products hi*hi + hi*lo + lo*hi keep 16 mantissa bits
        float sr_hi, sr_lo;
        split_bf16(sr[ln], sr_hi, sr_lo);
        const u32x4 sr_a = (h == 0) ? u32x4{pack2(sr_hi, sr_hi), pack2(sr_lo, 0.f), 0u, 0u} : u32x4{0u, 0u, 0u, 0u};

        // ---- production, by role (see GradCfg): writer wavefronts hash the writer's tables into phw; reader
        //      wavefronts project the reader and leave its per-bit masses (p, q, sech^2) in pm for the backward
        //      pass through the soft assignment; one more forms the in-tile term
        //      T^T[b][a] = Yw_b . Yr_a + sw_b * sr_a, masked, as MFMA operands for everybody
        if (intra && w < G::NW) {
            const int pg = w % G::NGW, pj = (w / G::NGW) % C::TPL, as = w / (G::NGW * C::TPL);
            constexpr int kShare = (1 << C::PHI) / G::AS;
            write_assignments<C, C::PST>(f32x16{0}, th * G::NGW + pg, ln, h, a.soft(), ln < nvalid, phw, pj, C::TPL, as * kShare,
                                         (as + 1) * kShare, nullptr, mw + ln * C::MS);
        }
        constexpr int kRd0 = INTRA ? G::RD0 : 0, kNr = INTRA ? G::NR : G::NR_NC, kRj = INTRA ? G::RJ : G::RJ_NC;
        if (w >= kRd0 && w < kRd0 + kNr) {
            const int pg = (w - kRd0) % G::NGW, rj = (w - kRd0) / G::NGW;
            const f32x16 zr = project<C>(wp, xr, th * G::NGW + pg, ln, h, UNIT ? nrm : nullptr);
#pragma unroll
            for (int j = 0; j < C::TPL; ++j) {
                if ((th * G::NGW + pg) * C::TPG + h * C::TPL + j >= C::L) break;
                if (j % kRj != rj) continue;
                float p[C::PP], q[C::PP], s2[C::PP], u[C::PP], zz[C::PP];
#pragma unroll
                for (int t = 0; t < C::PP; ++t) {
                    p[t] = q[t] = s2[t] = u[t] = 0.f;
                    zz[t] = t < C::P ? zr[zslot<C>(j, t)] : 0.f;
                }
                float *dst = pm + ((pg * C::TPG + h * C::TPL + j) * kTile + ln) * S::PMS;
                // (a padding table has zero statistics and zero cotangents: any finite masses will do)
                if (!C::PAD || (th * G::NGW + pg) * C::TPG + h * C::TPL + j < a.L_real) bit_masses<C>(zr, j, a.soft(), p, q, s2, u);
#pragma unroll
                for (int t = 0; t < C::PP; t += 4) {
                    *reinterpret_cast<float4 *>(dst + t) = float4{p[t], p[t + 1], p[t + 2], p[t + 3]};
                    *reinterpret_cast<float4 *>(dst + C::PP + t) = float4{q[t], q[t + 1], q[t + 2], q[t + 3]};
                    *reinterpret_cast<float4 *>(dst + 2 * C::PP + t) = float4{s2[t], s2[t + 1], s2[t + 2], s2[t + 3]};
                    *reinterpret_cast<float4 *>(dst + 3 * C::PP + t) = float4{u[t], u[t + 1], u[t + 2], u[t + 3]};
                    if (UNIT) *reinterpret_cast<float4 *>(dst + 4 * C::PP + t) = float4{zz[t], zz[t + 1], zz[t + 2], zz[t + 3]};
                }
            }
        }
        if (intra && w == G::TT) {
            f32x16 tt = {0};
            // both tiles keep their columns in the same (pair-interleaved) order, which is all a contraction needs
            const int yo = opaque(ln * C::XS + 8 * h), ywo = opaque(ln * C::YS + 8 * h);
#pragma unroll
            for (int s = 0; s < C::D / 16; ++s) tt = mma(lds128(yw + ywo + 16 * s), lds128(yr + yo + 16 * s), tt);
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
        // the next tile's loads are issued a whole step ahead and fly during everything below
        if (it + 1 < ntiles) fetch(it + 1);
        GRAD_PHASE(4)

        // ---- per 32-row tile of this wavefront: cotangent of the reader's assignments, transposed (lane = token,
        //      register v = bucket row r_own + 32 mr + acc_row(v, h)), then straight back through the corner
        //      softmax (Algorithm 1, step 4) in those registers: with w_c = phi_c dphi_c over the corners c of a
        //      table, m = sum_c w_c and, per bit t, G_t = sum of w_c over the corners on the bit's MINOR side
        //      (the side with the smaller mass min(p_t, q_t)).  The cotangent of u_t = tanh z_t is
        //      beta (E_t - m (p_t - q_t)) with E_t = sum_c v_{c,t} w_c; written as
        //      +-2 beta (small_t (m - G_t) - big_t G_t) it has no cancellation when the bit is saturated
        //      (small_t ~ 1e-7 at beta = 8), which the cotangent of beta needs.  Register v of lane half h is corner
        //      co + 8 (v/4 mod KM) + 4h + v%4 of table tl0 + (32 mr + 8 (v/4)) / R: bits 0,1 come from v, bit 2
        //      from h, bits 3.. from v, the bits above from the tile and the wavefront's share.  phi_c is the
        //      product over bits of p_t (bit set) or q_t (Section 3.3: the corner softmax factorises).
        float rec[G::TWW][8];          // [m, G_0 .. G_{P-1}] of the lane's token per table of the wavefront (lane partials)
#pragma unroll
        for (int i = 0; i < G::TWW; ++i) {
#pragma unroll
            for (int t = 0; t < 8; ++t) rec[i][t] = 0.f;
        }
#pragma unroll
        for (int mr = 0; mr < G::MTG; ++mr) {
            if (!has_rows) break;
            f32x16 dP;
            {
                // extra column first: sr_a * (A or dA)[r] with the masses before this tile
                float m_hi, m_lo;
                split_bf16(macc[mr] + __shfl_xor(macc[mr], 32, 64), m_hi, m_lo);
                const u32x4 mb = (h == 0) ? u32x4{pack2(m_hi, m_lo), pack2(m_hi, 0.f), 0u, 0u} : u32x4{0u, 0u, 0u, 0u};
                dP = mma(mb, sr_a, f32x16{0});
            }
            if (intra) {
#pragma unroll
                for (int s = 0; s < 2; ++s)
                    dP = mma(lds_tr_acc<true>(phw, C::PST, 16 * s, r_own + 32 * mr, ln, h), ttop[64 * s + lane], dP);
            }
            {
                const int yo = opaque(ln * C::XS + 8 * h);       // pair-interleaved columns: one 16-byte read per k-step
#pragma unroll
                for (int mtc = 0; mtc < C::NT; ++mtc) {
#pragma unroll
                    for (int s = 0; s < 2; ++s) {
                        const int cc = 32 * mtc + 16 * s;
                        dP = mma(acc_operand(ST[mr][mtc], s), lds128(yr + yo + cc), dP);
                    }
                }
            }
#pragma unroll
            for (int tw = 0; tw < G::TW; ++tw) {
                constexpr int kTilesPerTable = C::R >= 32 ? C::R / 32 : 1;
                const int ti = C::R >= 32 ? mr / kTilesPerTable : mr * G::TW + tw;   // table of the wavefront
                const int co = C::R >= 32 ? ro + 32 * (mr % kTilesPerTable) : 0;     // first corner of the tile in its table
                const float *src = pm + ((tl0 + ti) * kTile + ln) * S::PMS;
                float p[C::PP], q[C::PP];
#pragma unroll
                for (int t = 0; t < C::PP; t += 4) {
                    const float4 p4 = *reinterpret_cast<const float4 *>(src + t);
                    const float4 q4 = *reinterpret_cast<const float4 *>(src + C::PP + t);
                    p[t] = p4.x; p[t + 1] = p4.y; p[t + 2] = p4.z; p[t + 3] = p4.w;
                    q[t] = q4.x; q[t + 1] = q4.y; q[t + 2] = q4.z; q[t + 3] = q4.w;
                }
                float F = h ? p[2] : q[2];
#pragma unroll
                for (int t = 3 + G::MB; t < C::P; ++t) F *= ((co >> t) & 1) ? p[t] : q[t];
                const float Fl[4] = {F * q[0] * q[1], F * p[0] * q[1], F * q[0] * p[1], F * p[0] * p[1]};
                bool mn[C::PP];                    // the minor side of bit t is the value 1 (else the value 0)
#pragma unroll
                for (int t = 0; t < C::PP; ++t) mn[t] = p[t] < q[t];
                float m = 0.f, G0 = 0.f, G1 = 0.f, Gm[2] = {0.f, 0.f};
#pragma unroll
                for (int k = 0; k < G::KM; ++k) {
                    float mid = 1.f;
#pragma unroll
                    for (int b = 0; b < G::MB; ++b) mid *= ((k >> b) & 1) ? p[3 + b] : q[3 + b];
                    const int v0 = 4 * (tw * G::KM + k);
                    const float w0 = Fl[0] * dP[v0], w1 = Fl[1] * dP[v0 + 1], w2 = Fl[2] * dP[v0 + 2], w3 = Fl[3] * dP[v0 + 3];
                    const float s01 = w0 + w1, s23 = w2 + w3;
                    const float c = mid * (s01 + s23);
                    G0 = fmaf(mid, mn[0] ? w1 + w3 : w0 + w2, G0);
                    G1 = fmaf(mid, mn[1] ? s23 : s01, G1);
                    m += c;
#pragma unroll
                    for (int b = 0; b < G::MB; ++b) Gm[b] += (mn[3 + b] == (((k >> b) & 1) != 0)) ? c : 0.f;
                }
                // lane partials; bit 2 is the lane half, the bits above the tile's are uniform
                rec[ti][0] += m;
                rec[ti][1] += G0;
                rec[ti][2] += G1;
                rec[ti][3] += (mn[2] == (h != 0)) ? m : 0.f;
#pragma unroll
                for (int b = 0; b < G::MB; ++b) rec[ti][4 + b] += Gm[b];
#pragma unroll
                for (int t = 3 + G::MB; t < C::P; ++t) rec[ti][1 + t] += (mn[t] == (((co >> t) & 1) != 0)) ? m : 0.f;
            }
        }
        // the two lane halves hold the two values of bit 2: add them up
#pragma unroll
        for (int i = 0; i < G::TWW; ++i) {
#pragma unroll
            for (int t = 0; t <= C::P; ++t) rec[i][t] += __shfl_xor(rec[i][t], 32, 64);
        }
        if (G::WPT > 1 && has_rows && ro != 0) {
            // a later share of a table: hand the partial sums to the wavefront that owns the table's first share
            float *dst = part + ((w * kTile + ln) * 8 + 4 * h);
            *reinterpret_cast<float4 *>(dst) = float4{rec[0][4 * h], rec[0][4 * h + 1], rec[0][4 * h + 2], rec[0][4 * h + 3]};
        }
        GRAD_PHASE(5)
        // ---- statistics += Yw^T . phi_writer
        if (intra && has_rows) {
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                float4 g0 = {1.f, 1.f, 1.f, 1.f}, g1 = g0;          // SIDE 0: the extra column of [V | 1] is one
                if (SIDE == 1) {
                    g0 = *reinterpret_cast<const float4 *>(sw + 16 * s + 8 * h);
                    g1 = *reinterpret_cast<const float4 *>(sw + 16 * s + 8 * h + 4);
                }
                u32x4 ay[C::NT];
#pragma unroll
                for (int mtc = 0; mtc < C::NT; ++mtc) ay[mtc] = lds_tr_plain<true>(yw, C::YS, 16 * s, 32 * mtc, ln, h);
#pragma unroll
                for (int mr = 0; mr < G::MTG; ++mr) {
                    const u32x4 bp = lds_tr_plain<true>(phw, C::PST, 16 * s, r_own + 32 * mr, ln, h);
                    macc[mr] += SIDE == 1 ? wsum8(bp, g0, g1) : sum8(bp);
#pragma unroll
                    for (int mtc = 0; mtc < C::NT; ++mtc) ST[mr][mtc] = mma(ay[mtc], bp, ST[mr][mtc]);
                }
            }
        }
        GRAD_PHASE(10)
        GRAD_PHASE(6)
        __syncthreads();        // partial sums are visible; the tiles of this step are dead from here on
        GRAD_PHASE(7)

        // ---- finish per (token, table): du_t = +-2 beta (small_t (m - G_t) - big_t G_t),  dz_t = du_t (1 - tanh^2 z_t);
        //      lane half h' takes the padded projection slots 4h' .. 4h'+3
        // unit-norm option: dz is the cotangent of W xhat, so the reader's row gets dx = (g - xhat (xhat . g)) / |x| with
        // g = W^T dz and xhat . g = z . dz; dz is scaled by 1 / |x| here and this lane's share of z . dz is summed from the
        // bf16 values the matrix product below will see (which keeps dx orthogonal to x to fp32 accuracy)
        float radial = 0.f;
        if (has_rows && ro == 0) {
            const float rs = UNIT ? nrm[ln] : 1.f;
#pragma unroll
            for (int ti = 0; ti < G::TWW; ++ti) {
                if (4 * h >= C::PP) break;
                const int tl = tl0 + ti;
#pragma unroll
                for (int o = 1; o < G::WPT; ++o) {
                    const float *src = part + ((w + o) * kTile + ln) * 8;
                    const float4 p0 = *reinterpret_cast<const float4 *>(src);
                    const float4 p1 = *reinterpret_cast<const float4 *>(src + 4);
                    rec[ti][0] += p0.x; rec[ti][1] += p0.y; rec[ti][2] += p0.z; rec[ti][3] += p0.w;
                    rec[ti][4] += p1.x; rec[ti][5] += p1.y; rec[ti][6] += p1.z; rec[ti][7] += p1.w;
                }
                const float *src = pm + (tl * kTile + ln) * S::PMS + 4 * h;
                const float4 p4 = *reinterpret_cast<const float4 *>(src);
                const float4 q4 = *reinterpret_cast<const float4 *>(src + C::PP);
                const float4 s4 = *reinterpret_cast<const float4 *>(src + 2 * C::PP);
                const float4 u4 = *reinterpret_cast<const float4 *>(src + 3 * C::PP);
                const float pp[4] = {p4.x, p4.y, p4.z, p4.w}, qq[4] = {q4.x, q4.y, q4.z, q4.w};
                const float s2[4] = {s4.x, s4.y, s4.z, s4.w};
                const float uu[4] = {u4.x, u4.y, u4.z, u4.w};
                float dzv[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    // G of slot 4h + e is rec[1 + 4h + e]; slot 7 is padding (P <= 7) and has no entry
                    const float Gt = h ? (e < 3 ? rec[ti][e < 3 ? 5 + e : 0] : 0.f) : rec[ti][1 + e];
                    const bool minor1 = pp[e] < qq[e];                          // same predicate as where G was summed
                    const float small = minor1 ? pp[e] : qq[e], big = minor1 ? qq[e] : pp[e];
                    const float half = small * (rec[ti][0] - Gt) - big * Gt;
                    const float du = minor1 ? -2.f * half : 2.f * half;         // cotangent of u_t up to the factor beta
                    dzv[e] = a.beta * du * s2[e] * rs;                          // padded slots: p = q = s2 = 0
                    dbeta_acc = fmaf(du, uu[e], dbeta_acc);                     // ... and tanh = 0
                }
                // slot 4c.. of the lane-half hh's j-th table is projection row 8 (slots-per-table/4 * j + c) + 4 hh of its group
                const int gl = tl / C::TPG, tg = tl % C::TPG, hh = tg / C::TPL, j = tg % C::TPL;
                const int col = gl * 32 + 8 * ((C::PP / 4) * j + h) + 4 * hh;
                const u32x2 dzw = {pack2(dzv[0], dzv[1]), pack2(dzv[2], dzv[3])};
                *reinterpret_cast<u32x2 *>(dz + ln * S::DZS + col) = dzw;
                if (UNIT) {
                    const float4 z4 = *reinterpret_cast<const float4 *>(src + 4 * C::PP);
                    radial = fmaf(z4.x, bf_lo(dzw.x), radial);
                    radial = fmaf(z4.y, bf_hi(dzw.x), radial);
                    radial = fmaf(z4.z, bf_lo(dzw.y), radial);
                    radial = fmaf(z4.w, bf_hi(dzw.y), radial);
                }
            }
        }
        if (UNIT) {
            radial += __shfl_xor(radial, 32, 64);
            if (h == 0) rad[w * kTile + ln] = radial;
        }
        GRAD_PHASE(9)
        GRAD_PHASE(11)
        // (dX of this tile is formed after the next step's first barrier, see dx_stage)
        // no barrier here: the next step's loads-to-LDS touch none of dz, pm, part or the staging tiles, its production
        // (which rewrites pm) comes after the next barrier, and so does this tile's dX, which reads dz (rewritten only after
        // two more barriers) and, with the unit-norm option, this tile's reader rows and scales (the next step stores into
        // the other buffer, the step after that only after barriers the dX wavefronts take part in).
    }
    if (ntiles > 0) {
        __syncthreads();        // the last tile's dz is visible
        if (my_dx >= 0) {
            const int64_t tp = tile_t0(ntiles - 1);
            dx_stage(my_dx, tp, tile_nv(tp), tile_xr(ntiles - 1), tile_nrm(ntiles - 1));
        }
    }
    // ---- cotangent of beta: lanes -> wavefront (shuffles) -> workgroup (LDS, wavefront order) -> one workspace slot
    {
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) dbeta_acc += __shfl_xor(dbeta_acc, m, 64);
        __syncthreads();
        if (lane == 0) sr[w] = dbeta_acc;
        __syncthreads();
        if (tid == 0) {
            float s = 0.f;
            for (int i = 0; i < kWaves; ++i) s += sr[i];
            const int wgs = gridDim.x;                  // workgroups per (side, batch*head)
            a.dbeta_part[(static_cast<size_t>(SIDE) * gridDim.y + bh) * wgs + seg] = s;
        }
    }
    GRAD_PHASE_PRINT()
}

}  // namespace mfma
}  // namespace race
