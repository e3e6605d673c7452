// bf16 MFMA kernel family for RACE Attention on gfx950 (see mfma_common.h for the execution shape).
//
// Kernels
//   hash_kernel      projection and per-bit soft-hash masses of every row of Q and K, once per call: the "hashed rows"
//                    (one float per token, table and hyperplane) that every later pass rebuilds phi from.
//   scan_kernel      "totals" of the statistics per segment, then an exclusive prefix (forward) or
//                    suffix (backward) scan over segments turns them into segment-start states.
//   stream_kernel    one pass over a segment carrying statistics [L*R][d] in accumulator registers
//                    as tiles (bucket rows x head columns).  Modes:
//                      kTotalsKV  statistics of (phi_K, [V | 1])          (Algorithm 1, step 5)
//                      kTotalsQG  statistics of (phi_Q, read-out cotangents) for the backward pass
//                      kForward   Algorithm 2's loop / Algorithm 1's read-out: O and Den
//                      kGradV     the mirrored pass, right to left: dV
//   grad_kernel      (mfma_grad.h) the passes that contract over the head dimension: dQ and dK.
#include <hip/hip_runtime.h>

#include "internal.h"
#include <cstring>

#include "mfma_common.h"
#include "mfma_grad.h"

namespace race {
namespace mfma {

enum Mode { kTotalsKV = 0, kTotalsQG = 1, kForward = 2, kGradV = 3 };

// Developer aid: per-phase cycle counts of one workgroup, printed at kernel end (build with -DRACE_PHASE_TIMING).
#ifdef RACE_PHASE_TIMING
#define RACE_PHASE_DECL long long ph_t[12] = {0}; long long ph_last = clock64();
#define RACE_PHASE(i) { long long now_ = clock64(); ph_t[i] += now_ - ph_last; ph_last = now_; }
#define RACE_PHASE_PRINT(tag) if (blockIdx.x == 1 && blockIdx.y == 0 && (threadIdx.x & 63) == 0) \
    printf("%s mode %d wave %d tiles %d: load %lld prod %lld contr %lld upd %lld redw %lld epi %lld | waits %lld %lld %lld %lld %lld\n", tag, MODE, (int)(threadIdx.x >> 6), ntiles, \
           ph_t[0], ph_t[2], ph_t[4], ph_t[5], ph_t[7], ph_t[9], ph_t[1], ph_t[3], ph_t[6], ph_t[8], ph_t[10]);
#else
#define RACE_PHASE_DECL
#define RACE_PHASE(i)
#define RACE_PHASE_PRINT(tag)
#endif

// state element (bucket row r, column c) in the saved layout: B [LR][D] row-major, then A [LR]
template <class C>
__device__ __forceinline__ int state_b(int r, int c) { return r * C::D + c; }
template <class C>
__device__ __forceinline__ int state_a(int r) { return C::LR * C::D + r; }

template <class C>
__device__ __forceinline__ void load_projection_matrix(const KArgs &a, int head, bf16raw *wp)
{
    const bf16raw *src = a.Wp + static_cast<size_t>(head) * C::LPP * C::D;
    for (int c = threadIdx.x; c < C::LPP * C::CPR; c += kThreads) {
        const int row = c / C::CPR, ch = c % C::CPR;
        *reinterpret_cast<u32x4 *>(wp + row * C::XS + ch * 8) = *reinterpret_cast<const u32x4 *>(src + row * C::D + ch * 8);
    }
}

// ================================================================ hash_kernel
// Algorithm 1, steps 2-4 up to the per-bit masses, for every row of Q (blockIdx.z + first == 0) or K (== 1):
// z = W x on the matrix cores, then one float per (table, hyperplane), see bit_code().  No state is carried, so the
// grid is over token ranges: many small workgroups that hide each other's latencies, unlike the scans that follow.
template <class C>
struct HashLds {
    static constexpr int SLOTS = 4 / C::NG;                             // 32-token tiles per step (four wavefronts)
    static constexpr int TT = 32 * SLOTS;
    static constexpr int wp = 0;                                        // [LPP][XS] bf16
    static constexpr int x = wp + C::LPP * C::XS * 2;                   // [TT][XS] bf16 rows
    static constexpr int out = x + TT * C::XS * 2;                      // [TT][MS] fp32 hashed rows
    static constexpr int nx = out + TT * C::MS * 4;                     // [TT] fp32: 1 / |x| (unit-norm option)
    static constexpr int total = nx + TT * 4;
};
constexpr int kHashThreads = 256;
constexpr int kHashTokens = 512;        // tokens per workgroup (amortises the load of W)

template <class C, bool UNIT>
__global__ __launch_bounds__(kHashThreads) void hash_kernel(KArgs a, const bf16raw *Xq, const bf16raw *Xk, int first)
{
    using S = HashLds<C>;
    constexpr int TT = S::TT;
    extern __shared__ __attribute__((aligned(256))) unsigned char lds[];
    bf16raw *wp = reinterpret_cast<bf16raw *>(lds + S::wp);
    bf16raw *xs = reinterpret_cast<bf16raw *>(lds + S::x);
    float *out = reinterpret_cast<float *>(lds + S::out);
    float *nx = reinterpret_cast<float *>(lds + S::nx);
    const int which = static_cast<int>(blockIdx.z) + first;
    const int bh = blockIdx.y, head = bh % a.H;
    const int tid = threadIdx.x, w = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, ln = lane & 31, h = lane >> 5;
    const bf16raw *X = (which ? Xk : Xq) + static_cast<size_t>(bh) * a.N * C::D;
    float *M = (which ? a.Mk : a.Mq) + static_cast<size_t>(bh) * a.N * C::LP;
    {
        const bf16raw *src = a.Wp + static_cast<size_t>(head) * C::LPP * C::D;
        for (int c = tid; c < C::LPP * C::CPR; c += kHashThreads) {
            const int row = c / C::CPR, ch = c % C::CPR;
            *reinterpret_cast<u32x4 *>(wp + row * C::XS + ch * 8) = *reinterpret_cast<const u32x4 *>(src + row * C::D + ch * 8);
        }
    }
    const int64_t t_begin = static_cast<int64_t>(blockIdx.x) * kHashTokens;
    const int64_t t_end = (t_begin + kHashTokens < a.N) ? t_begin + kHashTokens : a.N;
    const Soft sf = a.soft();
    for (int64_t t0 = t_begin; t0 < t_end; t0 += TT) {
        const int nv = (t_end - t0 < TT) ? static_cast<int>(t_end - t0) : TT;
        // rows -> LDS (rows past the end repeat the last one: their results are not stored)
        for (int c = tid; c < TT * C::CPR; c += kHashThreads) {
            const int row = c / C::CPR, ch = c % C::CPR;
            const int rr = row < nv ? row : nv - 1;
            const u32x4 v = *reinterpret_cast<const u32x4 *>(X + (t0 + rr) * C::D + ch * 8);
            *reinterpret_cast<u32x4 *>(xs + row * C::XS + ch * 8) = v;
            if (UNIT) {
                const uint32_t xw[4] = {v.x, v.y, v.z, v.w};
                float ss = 0.f;
#pragma unroll
                for (int e = 0; e < 4; ++e) ss = dot2(xw[e], xw[e], ss);
#pragma unroll
                for (int m = C::CPR / 2; m >= 1; m >>= 1) ss += __shfl_xor(ss, m, 64);     // the chunks of a row sit in consecutive lanes
                if (ch == 0) nx[row] = __builtin_amdgcn_rsqf(fmaxf(ss, 1e-24f));
            }
        }
        __syncthreads();
        {
            const int slot = w / C::NG, g = w % C::NG;
            const f32x16 z = project<C>(wp, xs + slot * 32 * C::XS, g, ln, h, UNIT ? nx + slot * 32 : nullptr);
            float *orow = out + (slot * 32 + ln) * C::MS;
#pragma unroll
            for (int j = 0; j < C::TPL; ++j) {
                const int table = g * C::TPG + h * C::TPL + j;
                if (table >= C::L) break;
                const bool real_table = !C::PAD || table < sf.L;
#pragma unroll
                for (int t = 0; t < C::P; t += 2) {
                    float2 c2;
                    c2.x = (real_table && (!C::PAD || t < sf.P)) ? bit_code(z[zslot<C>(j, t)], sf.beta) : 0.f;
                    c2.y = (real_table && (!C::PAD || t + 1 < sf.P)) ? bit_code(z[zslot<C>(j, t + 1)], sf.beta) : 0.f;
                    *reinterpret_cast<float2 *>(orow + table * C::P + t) = c2;
                }
            }
        }
        __syncthreads();
        for (int c = tid; c < TT * C::MCH; c += kHashThreads) {
            const int row = c / C::MCH, ch = c % C::MCH;
            if (row < nv) {
                const float2 lo = *reinterpret_cast<const float2 *>(out + row * C::MS + ch * 4);
                const float2 hi = *reinterpret_cast<const float2 *>(out + row * C::MS + ch * 4 + 2);
                *reinterpret_cast<float4 *>(M + (t0 + row) * C::LP + ch * 4) = float4{lo.x, lo.y, hi.x, hi.y};
            }
        }
        // (the next step rewrites the row tile, which nobody reads any more, and `out` only after its first barrier)
    }
}

// ================================================================ totals_kernel
// Statistics of one segment from a zero start, 64 tokens per step (both halves of the workgroup hash
// 32 tokens each).  QG == 0: (phi_K, [V | 1]), Algorithm 1 step 5.  QG == 1: (phi_Q, [dO/e | -(dO.O)/e]),
// the statistics the key side of the backward pass reads.
template <class C>
struct TotalsLds {
    static constexpr int TT = 64;
    static constexpr int m = 0;                                         // [64][MS] fp32 hashed rows
    static constexpr int y = m + TT * C::MS * 4;                        // [64][YS] accumulated rows
    static constexpr int ph = y + TT * C::YS * 2;                       // [64][PST] assignments
    static constexpr int ge = ph + TT * C::PST * 2;                     // [64] fp32
    static constexpr int total = ge + TT * 4;
    static_assert(total <= 160 * 1024, "LDS budget");
};

// which column group carries the extra column of row tile mt (taking turns spreads the vector work over the wavefronts)
template <class C>
__device__ __forceinline__ bool mass_owner(int mt, int cg) { return mt % C::CG == cg; }

// M: the hashed rows of the tensor whose assignments feed the statistics (K forward, Q backward).
template <class C, int QG>
__global__ __launch_bounds__(kThreads, C::STREAM_WAVES_PER_SIMD)
void totals_kernel(KArgs a, const float *M, const bf16raw *Y, const bf16raw *Oin, const float *den_in)
{
    using S = TotalsLds<C>;
    constexpr int TT = S::TT;
    extern __shared__ __attribute__((aligned(256))) unsigned char lds[];
    float *ms = reinterpret_cast<float *>(lds + S::m);
    bf16raw *ys = reinterpret_cast<bf16raw *>(lds + S::y);
    bf16raw *ph = reinterpret_cast<bf16raw *>(lds + S::ph);
    float *ge_lds = reinterpret_cast<float *>(lds + S::ge);

    const int seg = blockIdx.x, bh = blockIdx.y;
    const int tid = threadIdx.x, w = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, ln = lane & 31, h = lane >> 5;
    const int rg = w % C::RG, cg = w / C::RG;
    const int r_own = rg * C::LRW, c_own = cg * C::DW;
    const size_t base = static_cast<size_t>(bh) * a.N * C::D;
    M += static_cast<size_t>(bh) * a.N * C::LP; Y += base;
    if (QG) { Oin += base; den_in += static_cast<size_t>(bh) * a.N; }
    float *st = a.state + (static_cast<size_t>(bh) * a.nseg + seg) * C::STATE;

    f32x16 Sacc[C::MT][C::NTW];
    float macc[C::MT];
#pragma unroll
    for (int mt = 0; mt < C::MT; ++mt) {
        macc[mt] = 0.f;
#pragma unroll
        for (int nt = 0; nt < C::NTW; ++nt) Sacc[mt][nt] = f32x16{0};
    }
    const int64_t t_begin = seg * a.seg_len;
    const int64_t t_end = (t_begin + a.seg_len < a.N) ? t_begin + a.seg_len : a.N;
    const int nsteps = static_cast<int>((t_end - t_begin + TT - 1) / TT);
    auto step_nv = [&](int64_t t0) { return (t_end - t0 < TT) ? static_cast<int>(t_end - t0) : TT; };

    MassChunks<C, TT> pre_m;
    RowChunks<C, TT> pre_y;
    CotChunks<C, TT> pre_c;
    auto fetch = [&](int it) {
        const int64_t t0 = t_begin + static_cast<int64_t>(it) * TT;
        const int nv = step_nv(t0);
        fetch_masses<C, TT>(M, t0, nv, pre_m);
        if (QG) fetch_cotangent<C, TT>(Y, Oin, den_in, t0, nv, pre_c);
        else fetch_rows<C, TT>(Y, t0, nv, pre_y);
    };
    if (nsteps > 0) fetch(0);

    for (int it = 0; it < nsteps; ++it) {
        const int64_t t0 = t_begin + static_cast<int64_t>(it) * TT;
        const int nvalid = step_nv(t0);
        store_masses<C, TT>(pre_m, ms);
        if (QG) store_cotangent<C, TT, C::YS>(pre_c, ys, ge_lds, a.L_real, nvalid);
        else store_rows<C, TT, C::YS>(pre_y, ys, nvalid);
        if (it + 1 < nsteps) fetch(it + 1);
        __syncthreads();
        {
            // wavefront = (token half, projection group, share of the group's tables)
            const int half = w / 4, g = w % C::NG, jq = (w % 4) / C::NG;
            write_assignments<C, C::PST>(f32x16{0}, g, half * 32 + ln, h, a.soft(), half * 32 + ln < nvalid, ph, jq, C::JSTEP, 0,
                                         1 << C::PHI, nullptr, ms + (half * 32 + ln) * C::MS);
        }
        __syncthreads();
#pragma unroll
        for (int s = 0; s < TT / 16; ++s) {
            u32x4 by[C::NTW];
#pragma unroll
            for (int nt = 0; nt < C::NTW; ++nt) by[nt] = lds_tr_plain(ys, C::YS, 16 * s, c_own + 32 * nt, ln, h);
            float4 g0 = {1.f, 1.f, 1.f, 1.f}, g1 = g0;
            if (QG) {
                g0 = *reinterpret_cast<const float4 *>(ge_lds + 16 * s + 8 * h);
                g1 = *reinterpret_cast<const float4 *>(ge_lds + 16 * s + 8 * h + 4);
            }
#pragma unroll
            for (int mt = 0; mt < C::MT; ++mt) {
                const u32x4 ap = lds_tr_plain<true>(ph, C::PST, 16 * s, r_own + 32 * mt, ln, h);
                if (mass_owner<C>(mt, cg))      // the extra column (bucket mass, or its cotangent): shared out over the column groups
                    macc[mt] += wsum8(ap, g0, g1);
#pragma unroll
                for (int nt = 0; nt < C::NTW; ++nt) Sacc[mt][nt] = mma(ap, by[nt], Sacc[mt][nt]);
            }
        }
        __syncthreads();
    }
#pragma unroll
    for (int mt = 0; mt < C::MT; ++mt) {
#pragma unroll
        for (int nt = 0; nt < C::NTW; ++nt) {
#pragma unroll
            for (int v = 0; v < 16; ++v)
                st[state_b<C>(r_own + 32 * mt + acc_row(v, h), c_own + 32 * nt + ln)] = Sacc[mt][nt][v];
        }
        const float tot = macc[mt] + __shfl_xor(macc[mt], 32, 64);
        if (mass_owner<C>(mt, cg) && h == 0) st[state_a<C>(r_own + 32 * mt + ln)] = tot;
    }
}

// ================================================================ stream_kernel
// One pass over a segment carrying the statistics as tiles S[bucket row][head column].
//   kForward: Algorithm 2's loop body (Algorithm 1's read-out when not causal): O and Den.
//   kGradV  : the mirrored pass, right to left, over the cotangent statistics: dV.
// "reader" = tensor whose assignments read the statistics (Q forward, K for dV), "writer" = tensor
// whose assignments feed them (K forward, Q for dV), Y = rows accumulated (V forward, dO/e for dV).
template <class C>
struct StreamLds {
    static constexpr int y = 0;                                         // [32][YS] bf16: accumulated rows
    static constexpr int mass = y + kTile * C::YS * 2;                  // [LR] fp32: bucket masses A before this tile, pair-interleaved
    static constexpr int dnp = mass + C::LR * 4;                        // [4][2][32] fp32: mass read-outs per reader wavefront and lane half
    static constexpr int mr = (dnp + 4 * 2 * kTile * 4 + 255) & ~255;   // [32][MS] fp32: hashed reader rows
    static constexpr int mw = mr + kTile * C::MS * 4;                   // [32][MS] fp32: hashed writer rows
    static constexpr int phr = (mw + kTile * C::MS * 4 + 15) & ~15;     // [32][PS] reader assignments
    static constexpr int phw = phr + kTile * C::PS * 2;                 // [32][PS] writer assignments
    static constexpr int endA = phw + kTile * C::PS * 2;
    // reduction over the bucket-row groups.  Where LDS allows it has bytes of its own: the epilogue of a tile then runs
    // next to the staging of the following tile instead of between two barriers of its own; otherwise it reuses the
    // bytes of the assignment tiles.
    static constexpr int RS = C::D + 4;                                 // fp32 row stride: D numerators, 1 normaliser part
    static constexpr int red_bytes = C::RG * kTile * RS * 4;            // [RG][32][RS] fp32
    static constexpr bool kOwnRed = ((endA + 255) & ~255) + red_bytes <= 160 * 1024;
    static constexpr int red = kOwnRed ? ((endA + 255) & ~255) : mr;
    static constexpr int total = kOwnRed ? red + red_bytes : (endA > mr + red_bytes ? endA : mr + red_bytes);
    static_assert(total <= 160 * 1024, "LDS budget");
};

// NC: the non-causal variant only (the in-tile term and the update are compiled out, which frees registers); the
// other variant reads the flag at run time (with the flag known to be set the compiler's schedule of the causal
// kernels needed more registers: the 128-register shapes spilled).
// Mr, Mw: the hashed rows of the reader and the writer tensor.
template <class C, int MODE, bool NC>
__global__ __launch_bounds__(kThreads, C::STREAM_WAVES_PER_SIMD)
void stream_kernel(KArgs a, const float *Mr, const float *Mw, const bf16raw *Y, const bf16raw *Oin,
                   const float *den_in, bf16raw *Out, float *den_out)
{
    using S = StreamLds<C>;
    extern __shared__ __attribute__((aligned(256))) unsigned char lds[];
    bf16raw *ytile = reinterpret_cast<bf16raw *>(lds + S::y);
    float *mass = reinterpret_cast<float *>(lds + S::mass);
    float *dnp = reinterpret_cast<float *>(lds + S::dnp);
    float *mr = reinterpret_cast<float *>(lds + S::mr);
    float *mw = reinterpret_cast<float *>(lds + S::mw);
    bf16raw *phr = reinterpret_cast<bf16raw *>(lds + S::phr);
    bf16raw *phw = reinterpret_cast<bf16raw *>(lds + S::phw);
    float *red = reinterpret_cast<float *>(lds + S::red);

    constexpr bool kReverse = (MODE == kGradV);
    const int seg = blockIdx.x, bh = blockIdx.y;
    const int tid = threadIdx.x, w = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, ln = lane & 31, h = lane >> 5;
    const int rg = w % C::RG, cg = w / C::RG;
    const int r_own = rg * C::LRW, c_own = cg * C::DW;
    const bool intra = NC ? false : a.causal != 0;    // causal: the tile's own keys take part

    const size_t base = static_cast<size_t>(bh) * a.N * C::D;
    Mr += static_cast<size_t>(bh) * a.N * C::LP; Mw += static_cast<size_t>(bh) * a.N * C::LP;
    Y += base; Out += base;
    if (MODE == kGradV) { Oin += base; den_in += static_cast<size_t>(bh) * a.N; }
    if (MODE == kForward) den_out += static_cast<size_t>(bh) * a.N;
    const float *st = a.state + (static_cast<size_t>(bh) * a.nseg + seg) * C::STATE;

    // statistics at the start of the segment
    f32x16 Sacc[C::MT][C::NTW];
    float macc[C::MT];                 // bucket masses (tiles mt % 2 == cg): per-half partial sums, lane n <-> row
#pragma unroll
    for (int mt = 0; mt < C::MT; ++mt) {
#pragma unroll
        for (int nt = 0; nt < C::NTW; ++nt) {
#pragma unroll
            for (int v = 0; v < 16; ++v)
                Sacc[mt][nt][v] = st[state_b<C>(r_own + 32 * mt + acc_row(v, h), c_own + 32 * nt + ln)];
        }
        // the bucket masses of tile mt are carried by column group mt % 2 (balances the vector work)
        macc[mt] = (MODE == kForward && mass_owner<C>(mt, cg) && h == 0) ? st[state_a<C>(r_own + 32 * mt + ln)] : 0.f;
        if (MODE == kForward && mass_owner<C>(mt, cg) && h == 0) mass[r_own + 32 * mt + il(ln)] = macc[mt];
    }

    const int64_t t_begin = seg * a.seg_len;
    const int64_t t_end = (t_begin + a.seg_len < a.N) ? t_begin + a.seg_len : a.N;
    const int ntiles = static_cast<int>((t_end - t_begin + kTile - 1) / kTile);
    auto tile_t0 = [&](int it) { return t_begin + static_cast<int64_t>(kReverse ? ntiles - 1 - it : it) * kTile; };
    auto tile_nv = [&](int64_t t0) { return (t_end - t0 < kTile) ? static_cast<int>(t_end - t0) : kTile; };

    // loads run one tile ahead of the arithmetic
    MassChunks<C, kTile> pre_r, pre_w;
    RowChunks<C, kTile> pre_y;
    CotChunks<C, kTile> pre_c;
    auto fetch = [&](int it) {
        const int64_t t0 = tile_t0(it);
        const int nv = tile_nv(t0);
        fetch_masses<C, kTile>(Mr, t0, nv, pre_r);
        if (intra) {
            fetch_masses<C, kTile>(Mw, t0, nv, pre_w);
            if (MODE == kGradV) fetch_cotangent<C, kTile>(Y, Oin, den_in, t0, nv, pre_c);
            else fetch_rows<C, kTile>(Y, t0, nv, pre_y);
        }
    };
    if (ntiles > 0) fetch(0);

    const float inv_tables = 1.0f / static_cast<float>(a.L_real);
    // ---- epilogue of one tile: thread = (token, pieces of 4 columns: 4i.. and, for d = 128, 64 + 4i..; consecutive
    //      threads read consecutive 16-byte pieces of the partials): sum, normalise, store
    auto epilogue = [&](int64_t t0, int nvalid) __attribute__((always_inline)) {
        {
        constexpr int NP = C::D / 64;                // pieces of 4 columns per thread
        const int tok = tid >> 4, c0 = (tid & 15) * 4;
        float acc[NP][4];
#pragma unroll
        for (int c = 0; c < NP; ++c) acc[c][0] = acc[c][1] = acc[c][2] = acc[c][3] = 0.f;
        float e = 0.f;
#pragma unroll
        for (int gg = 0; gg < 4; ++gg) {              // row groups (at most four) and the four reader wavefronts
            const float *src = red + (gg * kTile + tok) * S::RS;
            if (gg < C::RG) {
#pragma unroll
                for (int c = 0; c < NP; ++c) {
                    const float4 p4 = *reinterpret_cast<const float4 *>(src + c0 + 64 * c);
                    acc[c][0] += p4.x; acc[c][1] += p4.y; acc[c][2] += p4.z; acc[c][3] += p4.w;
                }
            }
            if (MODE == kForward) {
                const float dpart = dnp[gg * 64 + tok] + dnp[gg * 64 + 32 + tok];
                e += gg < C::RG ? src[C::D] + dpart : dpart;
            }
        }
        if (tok < nvalid) {
            const float scale = (MODE == kForward) ? (e > 0.f ? __builtin_amdgcn_rcpf(e) : 0.f) : 1.0f;   // e = 0: hard hash, empty buckets
            bf16raw *dst = Out + (t0 + tok) * C::D + c0;
#pragma unroll
            for (int c = 0; c < NP; ++c)
                *reinterpret_cast<u32x2 *>(dst + 64 * c) =
                    u32x2{pack2(acc[c][0] * scale, acc[c][1] * scale), pack2(acc[c][2] * scale, acc[c][3] * scale)};
            if (MODE == kForward && (tid & 15) == 0) den_out[t0 + tok] = e * inv_tables;
        }
    }
    };
    RACE_PHASE_DECL
    for (int it = 0; it < ntiles; ++it) {
        const int64_t t0 = tile_t0(it);
        const int nvalid = tile_nv(t0);
        // (the reduction buffer has bytes of its own: the previous tile's epilogue runs here, next to this tile's staging)
        if (S::kOwnRed && it > 0) {
            const int64_t tp = tile_t0(it - 1);
            epilogue(tp, tile_nv(tp));
        }

        // ---- registers -> LDS, then start the next tile's loads
        store_masses<C, kTile>(pre_r, mr);
        if (intra) {
            store_masses<C, kTile>(pre_w, mw);
            if (MODE == kGradV) store_cotangent<C, kTile, C::YS>(pre_c, ytile, nullptr, a.L_real, nvalid);
            else store_rows<C, kTile, C::YS>(pre_y, ytile, nvalid);
        }
        RACE_PHASE(0)
        __syncthreads();
        RACE_PHASE(1)

        // ---- production: wavefront = (side, projection group, share of the group's tables)
        {
            const int side = w / 4, g = w % C::NG, jq = (w % 4) / C::NG;
            if (side == 0) {
                const float dnl = write_assignments<C>(f32x16{0}, g, ln, h, a.soft(), true, phr, jq, C::JSTEP, 0, 1 << C::PHI,
                                                       MODE == kForward ? mass : nullptr, mr + ln * C::MS);
                if (MODE == kForward) dnp[w * 64 + lane] = dnl;       // this lane's tables' share of the normaliser
            } else if (intra) {
                write_assignments<C>(f32x16{0}, g, ln, h, a.soft(), ln < nvalid, phw, jq, C::JSTEP, 0, 1 << C::PHI, nullptr,
                                     mw + ln * C::MS);
            }
        }
        RACE_PHASE(2)
        __syncthreads();
        RACE_PHASE(3)

        // ---- contraction with the register-resident statistics (own bucket rows x own columns)
        f32x16 out[C::NTW];     // read-out, transposed: lane = reader token, register v = column acc_row(v, h) of the tile
        f32x16 sct = {0};       // in-tile kernel values, transposed: row = writer token, lane = reader token
        float rowsum = 0.f;     // in-tile part of the normaliser, reader token = ln
#pragma unroll
        for (int nt = 0; nt < C::NTW; ++nt) out[nt] = f32x16{0};
#pragma unroll
        for (int mt = 0; mt < C::MT; ++mt) {
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const int rr = r_own + 32 * mt + 16 * s + 8 * h;      // pair-interleaved corners: one 16-byte read
                const u32x4 ar = lds128(phr + ln * C::PS + rr);
#pragma unroll
                for (int nt = 0; nt < C::NTW; ++nt) out[nt] = mma(acc_operand(Sacc[mt][nt], s), ar, out[nt]);
                if (intra) {
                    const u32x4 aw = lds128(phw + ln * C::PS + rr);
                    sct = mma(aw, ar, sct);
                }
                RACE_SCHED_FENCE();
            }
        }
        if (intra) {
            // mask (writer token j = row, reader token i = lane), row sums, and (mask o kernel) . Y
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int j = acc_row(v, h);
                const bool keep = kReverse ? (j >= ln) : (j <= ln);
                sct[v] = keep ? sct[v] : 0.f;
                rowsum += sct[v];
            }
            rowsum += __shfl_xor(rowsum, 32, 64);
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const u32x4 ak = acc_operand(sct, s);
#pragma unroll
                for (int nt = 0; nt < C::NTW; ++nt)
                    out[nt] = mma(lds_tr_acc(ytile, C::YS, 16 * s, c_own + 32 * nt, ln, h), ak, out[nt]);
            }
        }
        if (intra) {
            RACE_PHASE(4)
            // ---- statistics += phi_writer^T . Y  (the read-out above used the old statistics)
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                u32x4 by[C::NTW];
#pragma unroll
                for (int nt = 0; nt < C::NTW; ++nt) by[nt] = lds_tr_plain(ytile, C::YS, 16 * s, c_own + 32 * nt, ln, h);
#pragma unroll
                for (int mt = 0; mt < C::MT; ++mt) {
                    const u32x4 ap = lds_tr_plain<true>(phw, C::PS, 16 * s, r_own + 32 * mt, ln, h);
                    if (MODE == kForward && mass_owner<C>(mt, cg)) macc[mt] += sum8(ap);
#pragma unroll
                    for (int nt = 0; nt < C::NTW; ++nt) Sacc[mt][nt] = mma(ap, by[nt], Sacc[mt][nt]);
                    RACE_SCHED_FENCE();
                }
            }
        }
        // the next tile's loads fly during the reduction and the epilogue (few registers are live there)
        if (it + 1 < ntiles) fetch(it + 1);
        RACE_PHASE(5)
        if (!S::kOwnRed) __syncthreads();       // every wavefront is done with the tiles of this step (whose bytes the partials reuse)
        RACE_PHASE(6)

        // ---- reduction over the bucket-row groups: partial read-outs through LDS, 16 bytes per store
        //      (a lane holds four consecutive columns of its token in registers 4k .. 4k+3)
        const int rbase = opaque((rg * kTile + ln) * S::RS + c_own + 4 * h);
#pragma unroll
        for (int nt = 0; nt < C::NTW; ++nt) {
#pragma unroll
            for (int k = 0; k < 4; ++k)
                *reinterpret_cast<float4 *>(red + rbase + 32 * nt + 8 * k) =
                    float4{out[nt][4 * k], out[nt][4 * k + 1], out[nt][4 * k + 2], out[nt][4 * k + 3]};
        }
        if (MODE == kForward) {
            // in-tile part of the normaliser: row sums of the masked kernel values (partial over this row group)
            if (cg == 0 && h == 0) red[(rg * kTile + ln) * S::RS + C::D] = rowsum;
            // masses after this tile, for the next tile's read-out
#pragma unroll
            for (int mt = 0; mt < C::MT; ++mt) {
                if (!mass_owner<C>(mt, cg)) continue;
                const float tot = macc[mt] + __shfl_xor(macc[mt], 32, 64);
                if (h == 0) mass[r_own + 32 * mt + il(ln)] = tot;
            }
        }
        RACE_PHASE(7)
        __syncthreads();
        RACE_PHASE(8)
        if (!S::kOwnRed) epilogue(t0, nvalid);
        RACE_PHASE(9)
        if (!S::kOwnRed) __syncthreads();
        RACE_PHASE(10)
    }
    if (S::kOwnRed && ntiles > 0) {
        const int64_t tp = tile_t0(ntiles - 1);
        epilogue(tp, tile_nv(tp));
    }
    RACE_PHASE_PRINT("stream")
}

// In-place scan over the segments of one (batch*head).  mode 0: exclusive prefix, 1: exclusive suffix,
// 2: every segment gets the total (non-causal).
__global__ void scan_kernel(float *state, int nseg, int elems, int mode)
{
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= elems) return;
    float *base = state + static_cast<size_t>(blockIdx.y) * nseg * elems + e;
    const size_t stride = static_cast<size_t>(elems);
    constexpr int U = 8;                 // segments in flight per thread: the loads of a group do not depend on the running sum
    float run = 0.f;
    if (mode == 2) {
        for (int s = 0; s < nseg; ++s) run += base[s * stride];
        for (int s = 0; s < nseg; ++s) base[s * stride] = run;
        return;
    }
    for (int s0 = 0; s0 < nseg; s0 += U) {
        float v[U];
#pragma unroll
        for (int k = 0; k < U; ++k) {
            const int s = mode == 0 ? s0 + k : nseg - 1 - (s0 + k);
            v[k] = (s0 + k < nseg) ? base[s * stride] : 0.f;
        }
#pragma unroll
        for (int k = 0; k < U; ++k) {
            const int s = mode == 0 ? s0 + k : nseg - 1 - (s0 + k);
            if (s0 + k < nseg) base[s * stride] = run;
            run += v[k];
        }
    }
}

// Totals over all segments of the problem's own buckets, written as A[row * a_stride] and
// Bsum[row * b_stride + c] with row = (bh * L_real + l) * R_real + r.  Real corner r of a real table sits at
// the compiled corner with all padding bits set.
template <class C>
__global__ void bucket_tap_kernel(const float *state, int nseg, int BH, int L_real, int P_real, float *A, float *Bsum,
                                  int a_stride, int b_stride)
{
    const int R_real = 1 << P_real, pad = (C::R - 1) & ~(R_real - 1);
    const size_t per = static_cast<size_t>(L_real) * R_real * (C::D + 1);
    const size_t i = blockIdx.x * static_cast<size_t>(blockDim.x) + threadIdx.x;
    if (i >= static_cast<size_t>(BH) * per) return;
    const size_t bh = i / per;
    const int e = static_cast<int>(i - bh * per);
    const int row = e / (C::D + 1), c = e % (C::D + 1), l = row / R_real, r = row % R_real;
    const int src = l * C::R + (r | pad);
    const int off = c < C::D ? src * C::D + c : C::LR * C::D + src;
    float run = 0.f;
    for (int s = 0; s < nseg; ++s) run += state[(bh * nseg + s) * C::STATE + off];
    const size_t dst = (bh * L_real + l) * R_real + r;
    if (c < C::D) Bsum[dst * b_stride + c] = run;
    else A[dst * a_stride] = run;
}

// Debug tap: hard codes and phi from the production step itself.
template <class C, bool UNIT>
__global__ __launch_bounds__(kThreads) void hash_tap_kernel(KArgs a, const bf16raw *X, uint8_t *codes, float *phi)
{
    extern __shared__ __attribute__((aligned(256))) unsigned char lds[];
    bf16raw *wp = reinterpret_cast<bf16raw *>(lds);
    bf16raw *x = wp + C::LPP * C::XS;
    bf16raw *ph = x + kTile * C::XS;
    float *nx = reinterpret_cast<float *>(ph + kTile * C::PS);      // [32] 1 / |x| (unit-norm option)
    const int bh = blockIdx.y, head = bh % a.H;
    const int tid = threadIdx.x, w = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, ln = lane & 31, h = lane >> 5;
    const int64_t t0 = static_cast<int64_t>(blockIdx.x) * kTile;
    const int nvalid = (a.N - t0 < kTile) ? static_cast<int>(a.N - t0) : kTile;
    const bf16raw *src = a.Wp + static_cast<size_t>(head) * C::LPP * C::D;
    for (int c = tid; c < C::LPP * C::CPR; c += kThreads) {
        const int row = c / C::CPR, ch = c % C::CPR;
        *reinterpret_cast<u32x4 *>(wp + row * C::XS + ch * 8) = *reinterpret_cast<const u32x4 *>(src + row * C::D + ch * 8);
    }
    {
        RowChunks<C, kTile> rows;
        fetch_rows<C, kTile>(X + static_cast<size_t>(bh) * a.N * C::D, t0, nvalid, rows);
        store_rows<C, kTile>(rows, x, nvalid);
        if (UNIT) store_row_scales<C, kTile>(rows, nx);
    }
    __syncthreads();
    if (w < C::NG) {
        const int g = w;
        const f32x16 z = project<C>(wp, x, g, ln, h, UNIT ? nx : nullptr);
        write_assignments<C>(z, g, ln, h, a.soft(), true, ph);
        if (ln < nvalid) {
#pragma unroll
            for (int j = 0; j < C::TPL; ++j) {
                const int table = g * C::TPG + h * C::TPL + j;
                if (table >= C::L || table >= a.L_real) break;
                unsigned code = 0;
#pragma unroll
                for (int t = 0; t < C::P; ++t) code |= (t < a.P_real && z[zslot<C>(j, t)] >= 0.f ? 1u : 0u) << t;
                codes[(static_cast<size_t>(bh) * a.N + t0 + ln) * a.L_real + table] = static_cast<uint8_t>(code);
            }
        }
    }
    __syncthreads();
    if (phi) {
        // the problem's own corners: real corner r of a real table is the compiled corner with all padding bits set
        const int R_real = 1 << a.P_real, LR_real = a.L_real * R_real, pad = (C::R - 1) & ~(R_real - 1);
        for (int i = tid; i < nvalid * LR_real; i += kThreads) {
            const int row = i / LR_real, lr = i % LR_real, src = (lr / R_real) * C::R + ((lr % R_real) | pad);
            phi[(static_cast<size_t>(bh) * a.N + t0 + row) * LR_real + lr] =
                __uint_as_float(static_cast<uint32_t>(ph[row * C::PS + il(src)]) << 16);
        }
    }
}

// Attainable matrix rate: four independent accumulators per wavefront, operands from registers only.
// NV > 0: every matrix instruction is followed by NV independent vector multiplies on registers of the same
// wavefront (eight dependency chains), the mix of a kernel that builds its operands with the vector ALU.
template <int NV>
__global__ __launch_bounds__(256) void calibration_mfma_kernel(int iters, float *sink)
{
    const uint32_t seed = 0x3F803F80u ^ (threadIdx.x & 1);          // bf16 values near one
    u32x4 a = {seed, seed, seed, seed}, b = {seed, seed, seed, seed};
    f32x16 c[4] = {f32x16{0}, f32x16{0}, f32x16{0}, f32x16{0}};
    float v[8];
    const float m = 1.0f + 1e-7f * static_cast<float>(threadIdx.x & 3);
#pragma unroll
    for (int r = 0; r < 8; ++r) v[r] = 1.0f + static_cast<float>(r);
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            c[k] = mma(a, b, c[k]);
            // (as instructions: plain C multiplies by a loop-invariant factor would be folded into one per chain)
#pragma unroll
            for (int r = 0; r < NV; ++r) asm volatile("v_mul_f32 %0, %0, %1" : "+v"(v[r % 8]) : "v"(m));
        }
    }
    const f32x16 cs = (c[0] + c[1]) + (c[2] + c[3]);
    float s = 0.f;
#pragma unroll
    for (int e = 0; e < 16; ++e) s += cs[e];
#pragma unroll
    for (int r = 0; r < 8; ++r) s += v[r];
    sink[static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x] = s;
}

}  // namespace mfma

// ================================================================================ host side
namespace {

using namespace mfma;

#define RACE_TRY(expr)                                   \
    do {                                                 \
        hipError_t e_ = (expr);                          \
        if (e_ != hipSuccess) return e_;                 \
    } while (0)

template <class K>
hipError_t allow_lds(K kernel, size_t bytes)
{
    return hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                               static_cast<int>(bytes));
}

template <class C>
KArgs make_kargs(const Plan &p, char *ws)
{
    KArgs a;
    a.H = p.H; a.nseg = p.nseg; a.causal = p.causal; a.N = p.N; a.seg_len = p.seg_len; a.beta = p.beta;
    a.L_real = p.L; a.P_real = p.P;
    a.Wp = reinterpret_cast<const bf16raw *>(ws + p.off_W);
    a.WpT = a.Wp + static_cast<size_t>(p.H) * C::LPP * C::D;
    a.state = reinterpret_cast<float *>(ws + p.off_stateA);
    a.Mq = reinterpret_cast<float *>(ws + p.off_massQ);
    a.Mk = reinterpret_cast<float *>(ws + p.off_massK);
    a.dbeta_part = reinterpret_cast<float *>(ws + p.off_dbeta);
    return a;
}

// Hashed rows of Q (first == 0) and/or K: `count` tensors starting with `first`.
template <class C>
hipError_t launch_hash(const Plan &p, KArgs a, const void *Q, const void *K, int first, int count, hipStream_t st)
{
    auto kern = p.unit_qk ? hash_kernel<C, true> : hash_kernel<C, false>;
    RACE_TRY(allow_lds(kern, HashLds<C>::total));
    ProfileScope prof("hash_rows", st);
    hipLaunchKernelGGL(kern, dim3(static_cast<unsigned>((p.N + kHashTokens - 1) / kHashTokens), p.BH, count), dim3(kHashThreads),
                       HashLds<C>::total, st, a, static_cast<const bf16raw *>(Q), static_cast<const bf16raw *>(K), first);
    return hipGetLastError();
}

template <class C, int QG>
hipError_t launch_totals(const Plan &p, KArgs a, const float *M, const void *Y, const void *O, const float *den_in,
                         hipStream_t st)
{
    auto kern = totals_kernel<C, QG>;
    RACE_TRY(allow_lds(kern, TotalsLds<C>::total));
    ProfileScope prof(QG ? "stream_totals_qg" : "stream_totals_kv", st);
    hipLaunchKernelGGL(kern, dim3(p.nseg, p.BH), dim3(kThreads), TotalsLds<C>::total, st, a, M,
                       static_cast<const bf16raw *>(Y), static_cast<const bf16raw *>(O), den_in);
    return hipGetLastError();
}

template <class C, int MODE>
hipError_t launch_stream(const Plan &p, KArgs a, const float *Mr, const float *Mw, const void *Y, const void *O,
                         const float *den_in, void *Out, float *den_out, hipStream_t st)
{
    static const char *const names[] = {"stream_totals_kv", "stream_totals_qg", "stream_forward", "stream_grad_v"};
    auto kern = p.causal ? stream_kernel<C, MODE, false> : stream_kernel<C, MODE, true>;
    RACE_TRY(allow_lds(kern, StreamLds<C>::total));
    ProfileScope prof(names[MODE], st);
    hipLaunchKernelGGL(kern, dim3(p.nseg, p.BH), dim3(kThreads), StreamLds<C>::total, st, a, Mr, Mw,
                       static_cast<const bf16raw *>(Y), static_cast<const bf16raw *>(O), den_in,
                       static_cast<bf16raw *>(Out), den_out);
    return hipGetLastError();
}

hipError_t launch_scan(const Plan &p, float *state, int elems, int mode, hipStream_t st)
{
    ProfileScope prof("segment_scan", st);
    hipLaunchKernelGGL(scan_kernel, dim3((elems + 255) / 256, p.BH), dim3(256), 0, st, state, p.nseg, elems, mode);
    return hipGetLastError();
}

template <class C>
hipError_t fwd_t(const Plan &p, const void *Q, const void *K, const void *V, void *O, float *den, char *ws, hipStream_t st)
{
    KArgs a = make_kargs<C>(p, ws);
    RACE_TRY((launch_hash<C>(p, a, Q, K, 0, 2, st)));
    RACE_TRY((launch_totals<C, 0>(p, a, a.Mk, V, nullptr, nullptr, st)));
    RACE_TRY(launch_scan(p, a.state, C::STATE, p.causal ? 0 : 2, st));
    RACE_TRY((launch_stream<C, kForward>(p, a, a.Mq, a.Mk, V, nullptr, nullptr, O, den, st)));
    return hipSuccess;
}

// dphi and the chain rule through the soft assignment and W (grad_kernel).
template <class C, int SIDE>
hipError_t launch_grad(const Plan &p, KArgs a, const void *Q, const void *K, const void *V, const void *O,
                       const float *den, const void *dO, void *dX, hipStream_t st)
{
    auto kern = p.causal ? (p.unit_qk ? grad_kernel<C, SIDE, true, true> : grad_kernel<C, SIDE, false, true>)
                         : (p.unit_qk ? grad_kernel<C, SIDE, true, false> : grad_kernel<C, SIDE, false, false>);
    const int lds = p.causal ? (p.unit_qk ? GradLds<C, true, true>::total : GradLds<C, false, true>::total)
                             : (p.unit_qk ? GradLds<C, true, false>::total : GradLds<C, false, false>::total);
    RACE_TRY(allow_lds(kern, lds));
    ProfileScope prof(SIDE == 0 ? "grad_q" : "grad_k", st);
    hipLaunchKernelGGL(kern, dim3(p.nseg, p.BH), dim3(kThreads), lds, st, a,
                       static_cast<const bf16raw *>(Q), static_cast<const bf16raw *>(K),
                       static_cast<const bf16raw *>(V), static_cast<const bf16raw *>(O), den,
                       static_cast<const bf16raw *>(dO), static_cast<bf16raw *>(dX));
    return hipGetLastError();
}

template <class C>
hipError_t bwd_t(const Plan &p, const void *Q, const void *K, const void *V, const void *O, const float *den,
                 const void *dO, void *dQ, void *dK, void *dV, float *dbeta, char *ws, hipStream_t st)
{
    KArgs a = make_kargs<C>(p, ws);
    KArgs b = a;
    b.state = reinterpret_cast<float *>(ws + p.off_stateB);
    // the hashed rows of Q and K and the statistics of (phi_K, [V | 1]) at segment starts (the forward leaves exactly
    // these behind: its scan is in place and its streaming pass only reads them); then the statistics of
    // (phi_Q, read-out cotangents) at segment ends
    if (!p.fwd_state_kept) {
        RACE_TRY((launch_hash<C>(p, a, Q, K, 0, 2, st)));
        RACE_TRY((launch_totals<C, 0>(p, a, a.Mk, V, nullptr, nullptr, st)));
        RACE_TRY(launch_scan(p, a.state, C::STATE, p.causal ? 0 : 2, st));
    }
    RACE_TRY((launch_totals<C, 1>(p, b, a.Mq, dO, O, den, st)));
    RACE_TRY(launch_scan(p, b.state, C::STATE, p.causal ? 1 : 2, st));
    RACE_TRY((launch_stream<C, kGradV>(p, b, a.Mk, a.Mq, dO, O, den, dV, nullptr, st)));
    RACE_TRY((launch_grad<C, 0>(p, a, Q, K, V, O, den, dO, dQ, st)));
    RACE_TRY((launch_grad<C, 1>(p, b, Q, K, V, O, den, dO, dK, st)));
    if (dbeta) RACE_TRY(reduce_dbeta(p, a.dbeta_part, dbeta, st));
    return hipSuccess;
}

template <class C>
hipError_t buckets_t(const Plan &p, const void *K, const void *V, float *A, float *Bsum, int a_stride, int b_stride,
                     char *ws, hipStream_t st)
{
    KArgs a = make_kargs<C>(p, ws);
    RACE_TRY((launch_hash<C>(p, a, nullptr, K, 1, 1, st)));
    RACE_TRY((launch_totals<C, 0>(p, a, a.Mk, V, nullptr, nullptr, st)));
    const size_t total = static_cast<size_t>(p.BH) * p.LR * (C::D + 1);
    hipLaunchKernelGGL(bucket_tap_kernel<C>, dim3(static_cast<unsigned>((total + 255) / 256)), dim3(256), 0, st, a.state,
                       p.nseg, p.BH, p.L, p.P, A, Bsum, a_stride, b_stride);
    return hipGetLastError();
}

template <class C>
hipError_t hash_t(const Plan &p, const void *X, uint8_t *codes, float *phi, char *ws, hipStream_t st)
{
    KArgs a = make_kargs<C>(p, ws);
    const size_t lds = (static_cast<size_t>(C::LPP) * C::XS + kTile * C::XS + kTile * C::PS) * 2 + kTile * 4;
    auto kern = p.unit_qk ? hash_tap_kernel<C, true> : hash_tap_kernel<C, false>;
    RACE_TRY(allow_lds(kern, lds));
    hipLaunchKernelGGL(kern, dim3(static_cast<unsigned>((p.N + kTile - 1) / kTile), p.BH), dim3(kThreads), lds, st, a,
                       static_cast<const bf16raw *>(X), codes, phi);
    return hipGetLastError();
}

uint16_t host_bf16(float x)
{
    uint32_t b;
    std::memcpy(&b, &x, 4);
    b += 0x7fffu + ((b >> 16) & 1u);
    return static_cast<uint16_t>(b >> 16);
}

// W (H, L*P, D) -> Wp (H, LPP, D) and WpT (H, D, LPP) in projection-group order: row rho of group g
// belongs to the lane half hh = (rho / 4) % 2; with a = rho / 8 and b = rho % 4 the half's slots (a, b)
// hold, for 8-padded tables, the half's table a/2 and hyperplane 4*(a%2) + b; for 4-padded tables, the half's
// table a and hyperplane b; the half's table j is table TPL*hh + j of the group.  Rows of padding (slots beyond
// the half's TPL tables, tables and hyperplanes the problem does not have) are zero.
template <class C>
void pack_t(const Plan &p, const float *W, void *image)
{
    uint16_t *wp = static_cast<uint16_t *>(image);
    uint16_t *wpt = wp + static_cast<size_t>(p.H) * C::LPP * C::D;
    for (int hd = 0; hd < p.H; ++hd) {
        for (int row = 0; row < C::LPP; ++row) {
            const int g = row / 32, rho = row % 32, a = rho / 8, hh = (rho / 4) % 2, b = rho % 4;
            const int j = (C::PP == 8) ? a / 2 : a;
            const int t = (C::PP == 8) ? 4 * (a % 2) + b : b;
            const int table = g * C::TPG + C::TPL * hh + j;
            for (int c = 0; c < C::D; ++c) {
                float v = 0.f;
                if (j < C::TPL && table < p.L && t < p.P) v = W[(static_cast<size_t>(hd) * p.LP + table * p.P + t) * C::D + c];
                const uint16_t bits = host_bf16(v);
                wp[(static_cast<size_t>(hd) * C::LPP + row) * C::D + c] = bits;
                wpt[(static_cast<size_t>(hd) * C::D + c) * C::LPP + row] = bits;
            }
        }
    }
}

// Dispatch over the compiled shapes.
#define RACE_SHAPES(X) RACE_MFMA_SHAPES(X)

}  // namespace

hipError_t calibration_mfma(int workgroups, int iters, int vector_ops, float *sink, hipStream_t st)
{
    switch (vector_ops) {
    case 0: hipLaunchKernelGGL(mfma::calibration_mfma_kernel<0>, dim3(workgroups), dim3(256), 0, st, iters, sink); break;
    case 4: hipLaunchKernelGGL(mfma::calibration_mfma_kernel<4>, dim3(workgroups), dim3(256), 0, st, iters, sink); break;
    case 8: hipLaunchKernelGGL(mfma::calibration_mfma_kernel<8>, dim3(workgroups), dim3(256), 0, st, iters, sink); break;
    case 16: hipLaunchKernelGGL(mfma::calibration_mfma_kernel<16>, dim3(workgroups), dim3(256), 0, st, iters, sink); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

bool mfma_pick(int d, int L, int P, int *Lc, int *Pc, int *pad)
{
    int best = 0;
#define X(DD, PP_, LL, PD)                                                                              \
    if (PD == 0 && d == DD && P == PP_ && L == LL) {                                                    \
        *Lc = LL; *Pc = PP_; *pad = 0;                                                                  \
        return true;                                                                                    \
    }
    RACE_SHAPES(X)
#undef X
#define X(DD, PP_, LL, PD)                                                                              \
    if (PD == 1 && d == DD && P <= PP_ && L <= LL && (best == 0 || LL * (1 << PP_) < best)) {           \
        best = LL * (1 << PP_);                                                                         \
        *Lc = LL; *Pc = PP_; *pad = 1;                                                                  \
    }
    RACE_SHAPES(X)
#undef X
    return best != 0;
}

size_t mfma_hashed_bytes(const Plan &p)
{
#define X(DD, PP_, LL, PD) if (p.d == DD && p.Pc == PP_ && p.Lc == LL && p.pad == PD) \
        return static_cast<size_t>(p.BH) * static_cast<size_t>(p.N) * Cfg<DD, PP_, LL, PD != 0>::LP * sizeof(float);
    RACE_SHAPES(X)
#undef X
    return 0;
}

size_t mfma_projection_bytes(const Plan &p)
{
#define X(DD, PP_, LL, PD) if (p.d == DD && p.Pc == PP_ && p.Lc == LL && p.pad == PD) return static_cast<size_t>(p.H) * Cfg<DD, PP_, LL, PD != 0>::LPP * DD * 2 * 2;
    RACE_SHAPES(X)
#undef X
    return 0;
}

void mfma_pack_projection(const Plan &p, const float *W, void *image)
{
#define X(DD, PP_, LL, PD) if (p.d == DD && p.Pc == PP_ && p.Lc == LL && p.pad == PD) return pack_t<Cfg<DD, PP_, LL, PD != 0>>(p, W, image);
    RACE_SHAPES(X)
#undef X
}

hipError_t mfma_fwd(const Plan &p, const void *Q, const void *K, const void *V, void *O, float *den, char *ws, hipStream_t st)
{
#define X(DD, PP_, LL, PD) if (p.d == DD && p.Pc == PP_ && p.Lc == LL && p.pad == PD) return fwd_t<Cfg<DD, PP_, LL, PD != 0>>(p, Q, K, V, O, den, ws, st);
    RACE_SHAPES(X)
#undef X
    return hipErrorNotSupported;
}

int mfma_dbeta_parts(const Plan &p)
{
    return p.nseg;
}

hipError_t mfma_bwd(const Plan &p, const void *Q, const void *K, const void *V, const void *O, const float *den,
                    const void *dO, void *dQ, void *dK, void *dV, float *dbeta, char *ws, hipStream_t st)
{
#define X(DD, PP_, LL, PD) if (p.d == DD && p.Pc == PP_ && p.Lc == LL && p.pad == PD) return bwd_t<Cfg<DD, PP_, LL, PD != 0>>(p, Q, K, V, O, den, dO, dQ, dK, dV, dbeta, ws, st);
    RACE_SHAPES(X)
#undef X
    return hipErrorNotSupported;
}

hipError_t mfma_hash(const Plan &p, const void *X_, uint8_t *codes, float *phi, char *ws, hipStream_t st)
{
#define X(DD, PP_, LL, PD) if (p.d == DD && p.Pc == PP_ && p.Lc == LL && p.pad == PD) return hash_t<Cfg<DD, PP_, LL, PD != 0>>(p, X_, codes, phi, ws, st);
    RACE_SHAPES(X)
#undef X
    return hipErrorNotSupported;
}

hipError_t mfma_buckets(const Plan &p, const void *K, const void *V, float *A, float *Bsum, int a_stride, int b_stride,
                        char *ws, hipStream_t st)
{
#define X(DD, PP_, LL, PD) if (p.d == DD && p.Pc == PP_ && p.Lc == LL && p.pad == PD) return buckets_t<Cfg<DD, PP_, LL, PD != 0>>(p, K, V, A, Bsum, a_stride, b_stride, ws, st);
    RACE_SHAPES(X)
#undef X
    return hipErrorNotSupported;
}

}  // namespace race
