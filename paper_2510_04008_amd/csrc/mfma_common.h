// Building blocks of the bf16 MFMA kernel family (gfx950): compile-time shapes, LDS tile layouts,
// operand loads, the projection + soft-assignment "production" step.
//
// Execution shape.  One workgroup of eight wavefronts (two per SIMD, 256 registers each) owns one
// (batch*head, segment) and walks its tokens in tiles of 32.  The bucket statistics of all L tables,
// [L*R][d] fp32 (B of Algorithm 1, step 5; A is kept beside it), never leave the register file: every
// wavefront holds an eighth of them as 32x32 MFMA accumulator tiles (stream kernels: a quarter of the
// bucket rows x half of the columns; grad kernel: an eighth of the bucket rows x all columns, transposed).
// Per tile the workgroup
//   1. projects the 32 query and key rows on all L*P hyperplanes (MFMA) and turns the projections
//      into soft assignments phi (vector ALU), written as bf16 tiles to LDS;
//   2. contracts them with the register-resident statistics and with each other (MFMA).
// MFMA 32x32x16 bf16 register layouts used throughout (lane = 32*h + n):
//   A operand: row n of A, columns 8h..8h+7 of the 16-wide k-step;   B operand: column n of B, rows 8h..8h+7;
//   C/D      : column n, rows 8*(v/4) + 4h + v%4 for register v = 0..15.
// An accumulator tile is fed back as a B operand without touching LDS: registers 8s..8s+7 of the
// tile, packed to bf16, are the B operand of k-step s if k-slot (h, e) is taken to mean row
// 16s + 8*(e/4) + 4h + e%4.  The other operand must use the same k order; tiles that are contracted
// against such operands keep their feature dimension "pair-interleaved" in LDS (il()): inside every
// group of 16 features the two middle blocks of 4 are swapped, so that the 8 features a lane needs
// are one aligned 16-byte read.
// LDS bank arithmetic as measured on gfx950 (64 banks of 4 bytes, 256 bytes per clock for reads: 16-byte
// accesses go 16 lanes at a time, 8-byte ones 32 lanes): rows read 16 bytes per lane want a row stride of
// 4 mod 64 words; tiles read through the transposing 8-byte loads (per 16 lanes 4 rows x 32 bytes, the
// next 16 lanes 32 bytes further) want 16 mod 32 words.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace race {
namespace mfma {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef uint16_t bf16raw;

constexpr int kWaves = 8;
constexpr int kThreads = 64 * kWaves;
constexpr int kRowGroups = 4;  // most row groups a workgroup's statistics are split into (stream kernels)
constexpr int kTile = 32;      // tokens per tile

// PAD_: the instantiation also serves problems with fewer tables and hyperplanes than its shape (see Soft).
template <int D_, int P_, int L_, bool PAD_ = false>
struct Cfg {
    static constexpr int D = D_, P = P_, L = L_;
    static constexpr bool PAD = PAD_;
    static constexpr int R = 1 << P, LR = L * R;
    static constexpr int PP = P > 4 ? 8 : 4;            // hyperplanes per table, padded
    // tables per 32-row projection group: as many as fit, or (shapes with fewer tables) the tables there are, spread
    // over both lane halves; the group's remaining rows are padding
    static constexpr int TPG = (32 / PP < L + (L & 1)) ? 32 / PP : L + (L & 1);
    static constexpr int TPL = TPG / 2;                 // tables per lane (per half-wave)
    static constexpr int NG = (L + TPG - 1) / TPG;      // projection groups
    static constexpr int LPP = NG * 32;                 // padded projection rows
    // stream kernels: wavefront w owns bucket-row group w % RG and column group w / RG (four row groups x two
    // column groups, or two x four when there are only 64 bucket rows)
    static constexpr int RG = LR / 32 >= kRowGroups ? kRowGroups : LR / 32;
    static constexpr int CG = kWaves / RG;
    static constexpr int LRW = LR / RG;                 // bucket rows of one row group
    static constexpr int MT = LRW / 32;                 // 32-row tiles of bucket rows per row group
    static constexpr int NT = D / 32;                   // 32-column tiles of the head dimension
    static constexpr int NTW = NT / CG;                 // column tiles per wavefront
    static constexpr int DW = D / CG;                   // columns per wavefront
    // wavefronts per SIMD the stream and totals kernels are compiled for: shapes with at most two accumulator
    // tiles of statistics and one column tile per wavefront fit 128 registers and leave room for a second workgroup
    // on the CU, whose phases interleave with the first one's (measured: with two column tiles the kernels spill
    // at 128 registers and lose more than the second workgroup gains)
    static constexpr int STREAM_WAVES_PER_SIMD = (MT * NTW <= 2 && NTW == 1) ? 4 : 2;
    static constexpr int LRG = LR / kWaves;             // bucket rows per wavefront (grad kernel)
    static constexpr int MTG = LRG / 32;                // 32-row tiles per wavefront (grad kernel)
    static constexpr int JSTEP = 4 / NG;                // wavefronts that share one projection group
    static constexpr int PLO = P < 3 ? P : 3, PHI = P - PLO;
    static constexpr int CPR = D / 8;                   // 16-byte chunks per row
    // LDS row strides, in bf16 elements (rows stay 16-byte aligned; the pad staggers banks)
    static constexpr int XS = D + 8;                    // [token][d] tiles and W rows, read by rows
    static constexpr int YS = D + 32;                   // [token][d] tiles read through transposing loads
    static constexpr int PS = LR + 8;                   // [token][L*R] assignment tiles, read by rows
    static constexpr int PST = LR + 16;                 // ... read through transposing loads only (a compromise:
                                                        // 16-byte row writes and transposing reads both 2-way at most)
    static constexpr int ZS = LPP + 8;                  // [token][padded projection] tiles
    static constexpr int STATE = LR * (D + 1);          // floats per saved state: B [LR][D] then A [LR]
    // hashed form of a row (see bit_code()): one float per (table, hyperplane), L * P per token
    static constexpr int LP = L * P;
    static constexpr int MS = LP + 2;                   // [token][LP] tiles of them in LDS: an even stride whose half is odd keeps the 8-byte
                                                        // reads of 32 consecutive tokens on distinct banks
    static constexpr int MCH = LP / 4;                  // 16-byte chunks per token
    static_assert(P % 2 == 0 && LP % 4 == 0 && (MS / 2) % 2 == 1, "hashed rows are read as pairs of floats");
    static_assert(RG >= 1 && LR % (32 * RG) == 0 && NT % CG == 0 && NTW >= 1, "bucket rows and columns over the wavefronts");
    static_assert(D % 64 == 0 && P >= 4, "shape (assignments are written for pairs of high-bit indices)");
    static_assert(4 % NG == 0 && NG <= 4, "projection groups must divide four wavefronts");
};

// Scheduling fence: keeps the instruction scheduler from hoisting the loads and conversions of later
// loop iterations (and with them dozens of live registers) above this point.
#define RACE_SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)

// Hides the value of an index from the optimiser inside a loop body, so that the dozens of addresses
// derived from it (index + constant) are folded into instruction offsets instead of being hoisted out of
// the loop as separate loop-invariant registers (which then spill).
__device__ __forceinline__ int opaque(int x)
{
    asm volatile("" : "+v"(x));
    return x;
}

// The soft assignment's run-time parameters.  A compiled shape <d, P, L> also serves smaller problems
// (tables L_real <= L, hyperplanes P_real <= P): tables beyond L_real get zero assignments, and a hyperplane
// beyond P_real is a bit whose mass sits entirely on its +1 side, so that the 2^P_real real corners are the
// corners of the compiled hypercube with all padding bits set.
struct Soft {
    float beta;
    int L, P;
};

// kernel arguments common to the family
struct KArgs {
    int H, nseg, causal;
    int64_t N, seg_len;
    float beta;
    int L_real, P_real;    // the problem's tables and hyperplanes (<= the compiled shape's)
    __host__ __device__ Soft soft() const { return Soft{beta, L_real, P_real}; }
    const bf16raw *Wp;     // (H, LPP, D) bf16, rows in projection-group order
    const bf16raw *WpT;    // (H, D, LPP) bf16
    float *state;          // (BH, nseg, STATE) fp32
    float *Mq, *Mk;        // (BH, N, L * P) fp32: the hashed rows of Q and K (hash_kernel writes them, every later pass reads them)
    float *dbeta_part;     // (2, BH, workgroups per head-batch) fp32: partial cotangents of beta (backward only)
};

// ---------------------------------------------------------------- small helpers
__device__ __forceinline__ uint32_t pack2(float lo, float hi)
{
    f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
__device__ __forceinline__ float bf_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

__device__ __forceinline__ f32x16 mma(u32x4 a, u32x4 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c,
                                                   0, 0, 0);
}
__device__ __forceinline__ u32x4 lds128(const bf16raw *p) { return *reinterpret_cast<const u32x4 *>(p); }
__device__ __forceinline__ u32x4 lds64x2(const bf16raw *p0, const bf16raw *p1)
{
    const u32x2 a = *reinterpret_cast<const u32x2 *>(p0), b = *reinterpret_cast<const u32x2 *>(p1);
    return u32x4{a.x, a.y, b.x, b.y};
}
// accumulator registers 8s..8s+7 as a bf16 B (or A) operand
__device__ __forceinline__ u32x4 acc_operand(const f32x16 &t, int s)
{
    return s == 0 ? u32x4{pack2(t[0], t[1]), pack2(t[2], t[3]), pack2(t[4], t[5]), pack2(t[6], t[7])}
                  : u32x4{pack2(t[8], t[9]), pack2(t[10], t[11]), pack2(t[12], t[13]), pack2(t[14], t[15])};
}
// fp32 value as a bf16 pair (hi, lo) with hi + lo = x to 16 mantissa bits
__device__ __forceinline__ void split_bf16(float x, float &hi, float &lo)
{
    hi = bf_lo(pack2(x, 0.f));
    lo = x - hi;
}
// a.lo * b.lo + a.hi * b.hi + c on words of two bf16 (v_dot2c_f32_bf16: exact products, fp32 sums)
__device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float c)
{
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a), __builtin_bit_cast(bf16x2, b), c, false);
}
constexpr uint32_t kOnePair = 0x3F803F80u;     // (1.0, 1.0)
// sum of the eight bf16 of v
__device__ __forceinline__ float sum8(u32x4 v)
{
    return dot2(v.y, kOnePair, dot2(v.x, kOnePair, 0.f)) + dot2(v.w, kOnePair, dot2(v.z, kOnePair, 0.f));
}
// sum of v_i g_i over the eight bf16 of v with fp32 weights.  (Plain multiply-adds: with the weights as bf16 (hi, lo)
// pairs and eight packed dot instructions the totals and gradient kernels measured 1-4 % slower.)
__device__ __forceinline__ float wsum8(u32x4 v, float4 g0, float4 g1)
{
    return bf_lo(v.x) * g0.x + bf_hi(v.x) * g0.y + bf_lo(v.y) * g0.z + bf_hi(v.y) * g0.w +
           bf_lo(v.z) * g1.x + bf_hi(v.z) * g1.y + bf_lo(v.w) * g1.z + bf_hi(v.w) * g1.w;
}
// row of accumulator register v for lane half h
__device__ __forceinline__ int acc_row(int v, int h) { return 8 * (v >> 2) + 4 * h + (v & 3); }
// pair-interleaved position of feature c: bits 2 and 3 of the index swapped
__device__ __forceinline__ constexpr int il(int c) { return (c & ~12) | ((c & 4) << 1) | ((c & 8) >> 1); }

// ---------------------------------------------------------------- transposing operand reads
// MFMA operand whose k index runs along the ROWS of a row-major LDS tile M[k][n] (stride in elements):
// lane (n, h) gets column n0 + n, rows k0a..k0a+3 then k0b..k0b+3.  Built from two ds_read_b64_tr_b16:
// within a block of 16 lanes, lane i supplies the address of a 4-element row chunk and receives element
// i%4 of the chunks of lanes i/4, i/4 + 4, i/4 + 8, i/4 + 12; with chunk (row i/4, columns 4(i%4)..) per
// lane that is column i of four consecutive rows.
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef s16x4 __attribute__((address_space(3))) lds_s16x4;
// IL: the tile's columns are pair-interleaved (the chunk of logical columns 4c.. sits at 4 * swap(c)).
template <bool IL = false>
__device__ __forceinline__ u32x4 lds_tr8(const bf16raw *M, int stride, int k0a, int k0b, int n0, int ln)
{
    const int sub = ln & 15;
    const int chunk = IL ? (((sub & 1) << 1) | ((sub >> 1) & 1)) : (sub & 3);
    const bf16raw *p = M + (sub >> 2) * stride + n0 + 16 * (ln >> 4) + 4 * chunk;
    const s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(p + k0a * stride));
    const s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(p + k0b * stride));
    const u32x2 ua = __builtin_bit_cast(u32x2, a), ub = __builtin_bit_cast(u32x2, b);
    return u32x4{ua.x, ua.y, ub.x, ub.y};
}
// k-slots in plain order (rows k0 + 8h + 0..7) or in accumulator order (pairs with acc_operand)
template <bool IL = false>
__device__ __forceinline__ u32x4 lds_tr_plain(const bf16raw *M, int stride, int k0, int n0, int ln, int h)
{
    return lds_tr8<IL>(M, stride, k0 + 8 * h, k0 + 8 * h + 4, n0, ln);
}
template <bool IL = false>
__device__ __forceinline__ u32x4 lds_tr_acc(const bf16raw *M, int stride, int k0, int n0, int ln, int h)
{
    return lds_tr8<IL>(M, stride, k0 + 4 * h, k0 + 8 + 4 * h, n0, ln);
}

// ---------------------------------------------------------------- global -> registers -> LDS tiles
// A tile of ROWS rows is ROWS*CPR chunks of 16 bytes; thread t owns chunks t, t + 512, ...  Loads are
// issued ahead of use (fetch) and written to LDS later (store), so that HBM latency overlaps arithmetic.
// (NTHR: the threads that share the tile, the first NTHR of the workgroup)
template <class C, int ROWS, int NTHR = kThreads>
struct RowChunks {
    static constexpr int N = (ROWS * C::CPR + NTHR - 1) / NTHR;
    u32x4 v[N];
};

// Every lane loads, unconditionally: rows past the end of the tile (nvalid >= 1 rows are real) re-read the last real
// row and are zeroed when they are stored.  (A load under a condition, into registers cleared first, makes the
// compiler wait for every load in flight before the clearing moves: the loads of a tile would complete one by one.)
// SBASE: the address as a uniform base plus a 32-bit byte offset per lane, which lets the loads take their base from
// scalar registers (10-15 vector registers fewer in the gradient kernel, which needs them; the stream and totals
// kernels measured 1-4 % slower with it and keep the plain form).
template <class C, int ROWS, bool SBASE = false, int NTHR = kThreads>
__device__ __forceinline__ void fetch_rows(const bf16raw *X, int64_t t0, int nvalid, RowChunks<C, ROWS, NTHR> &r)
{
    const char *base = reinterpret_cast<const char *>(X + t0 * C::D);
#pragma unroll
    for (int k = 0; k < RowChunks<C, ROWS, NTHR>::N; ++k) {
        const int c = threadIdx.x + k * NTHR, row = c / C::CPR, ch = c % C::CPR;
        const int rr = row < nvalid ? row : nvalid - 1;
        if (SBASE) r.v[k] = *reinterpret_cast<const u32x4 *>(base + static_cast<uint32_t>((rr * C::D + ch * 8) * 2));
        else r.v[k] = *reinterpret_cast<const u32x4 *>(X + (t0 + rr) * C::D + ch * 8);
    }
}

// One 16-byte chunk (columns 8ch .. 8ch+7) into row-major tile `dst` with row stride STRIDE; IL: pair-interleaved
// columns (the chunk's two blocks of 4 land 8 positions apart).
template <int STRIDE, bool IL>
__device__ __forceinline__ void store_chunk(bf16raw *dst, int row, int ch, u32x4 v)
{
    if (IL) {
        bf16raw *p = dst + row * STRIDE + 16 * (ch >> 1) + 4 * (ch & 1);
        *reinterpret_cast<u32x2 *>(p) = u32x2{v.x, v.y};
        *reinterpret_cast<u32x2 *>(p + 8) = u32x2{v.z, v.w};
    } else {
        *reinterpret_cast<u32x4 *>(dst + row * STRIDE + ch * 8) = v;
    }
}

// nvalid: rows of the tile that exist; the others are stored as zeros.
template <class C, int ROWS, int STRIDE = C::XS, bool IL = false, int NTHR = kThreads>
__device__ __forceinline__ void store_rows(const RowChunks<C, ROWS, NTHR> &r, bf16raw *dst, int nvalid)
{
    const int tid = opaque(static_cast<int>(threadIdx.x));       // keeps the tile addresses out of long-lived registers
#pragma unroll
    for (int k = 0; k < RowChunks<C, ROWS, NTHR>::N; ++k) {
        const int c = tid + k * NTHR, row = c / C::CPR, ch = c % C::CPR;
        const bool real = row < nvalid;
        const u32x4 v = {real ? r.v[k].x : 0u, real ? r.v[k].y : 0u, real ? r.v[k].z : 0u, real ? r.v[k].w : 0u};
        if (row < ROWS) store_chunk<STRIDE, IL>(dst, row, ch, v);
    }
}

// Hashed rows: a tile of ROWS tokens is ROWS * C::MCH chunks of 16 bytes, contiguous in memory; thread t owns chunks
// t, t + 512, ... (most shapes: one, and not every thread has one).
template <class C, int ROWS, int NTHR = kThreads>
struct MassChunks {
    static constexpr int N = (ROWS * C::MCH + NTHR - 1) / NTHR;
    u32x4 v[N];
};
// SBASE: a uniform base plus a 32-bit byte offset per lane (see fetch_rows).
template <class C, int ROWS, bool SBASE = false, int NTHR = kThreads>
__device__ __forceinline__ void fetch_masses(const float *M, int64_t t0, int nvalid, MassChunks<C, ROWS, NTHR> &r)
{
    const char *base = reinterpret_cast<const char *>(M + t0 * C::LP);
#pragma unroll
    for (int k = 0; k < MassChunks<C, ROWS, NTHR>::N; ++k) {
        const int c = threadIdx.x + k * NTHR, row = c / C::MCH, ch = c % C::MCH;
        const int rr = row < nvalid ? row : nvalid - 1;         // (rows past the end re-read the last real row; their phi is zeroed)
        if (SBASE) r.v[k] = *reinterpret_cast<const u32x4 *>(base + static_cast<uint32_t>((rr * C::LP + ch * 4) * 4));
        else r.v[k] = *reinterpret_cast<const u32x4 *>(M + (t0 + rr) * C::LP + ch * 4);
    }
}
template <class C, int ROWS, int NTHR = kThreads>
__device__ __forceinline__ void store_masses(const MassChunks<C, ROWS, NTHR> &r, float *dst)
{
    const int tid = opaque(static_cast<int>(threadIdx.x));
#pragma unroll
    for (int k = 0; k < MassChunks<C, ROWS, NTHR>::N; ++k) {
        const int c = tid + k * NTHR, row = c / C::MCH, ch = c % C::MCH;
        if (row < ROWS) {
            u32x2 *p = reinterpret_cast<u32x2 *>(dst + row * C::MS + ch * 4);
            p[0] = u32x2{r.v[k].x, r.v[k].y};
            p[1] = u32x2{r.v[k].z, r.v[k].w};
        }
    }
}

// Unit-norm option (the setting |Q_i| = |K_j| = 1 of Theorem 1's proof): scale[row] = 1 / max(|x_row|, 1e-12) for the
// rows held in r, from the fp32 sum of squares of the stored elements.  (Rows past the end of a tile hold a copy of
// the last real row.)
template <class C, int ROWS>
__device__ __forceinline__ void store_row_scales(const RowChunks<C, ROWS> &r, float *scale)
{
    const int tid = opaque(static_cast<int>(threadIdx.x));
#pragma unroll
    for (int k = 0; k < RowChunks<C, ROWS>::N; ++k) {
        const int c = tid + k * kThreads, row = c / C::CPR, ch = c % C::CPR;
        const uint32_t xw[4] = {r.v[k].x, r.v[k].y, r.v[k].z, r.v[k].w};
        float ss = 0.f;
#pragma unroll
        for (int e = 0; e < 4; ++e) ss = dot2(xw[e], xw[e], ss);
        // the CPR threads of one row are consecutive lanes
#pragma unroll
        for (int m = C::CPR / 2; m >= 1; m >>= 1) ss += __shfl_xor(ss, m, 64);
        if (ch == 0 && row < ROWS) scale[row] = __builtin_amdgcn_rsqf(fmaxf(ss, 1e-24f));
    }
}

// Read-out cotangent rows: gn = dO / e (e = L * Den) as bf16 rows, ge[row] = -(gn . O) as fp32 (= -(dO . O) / e).
template <class C, int ROWS, int NTHR = kThreads>
struct CotChunks {
    RowChunks<C, ROWS, NTHR> g, o;
    float den[RowChunks<C, ROWS, NTHR>::N];
};

template <class C, int ROWS, bool SBASE = false, int NTHR = kThreads>
__device__ __forceinline__ void fetch_cotangent(const bf16raw *dO, const bf16raw *O, const float *den, int64_t t0,
                                                int nvalid, CotChunks<C, ROWS, NTHR> &r)
{
    fetch_rows<C, ROWS, SBASE, NTHR>(dO, t0, nvalid, r.g);
    fetch_rows<C, ROWS, SBASE, NTHR>(O, t0, nvalid, r.o);
    const char *dbase = reinterpret_cast<const char *>(den + t0);
#pragma unroll
    for (int k = 0; k < RowChunks<C, ROWS, NTHR>::N; ++k) {
        const int row = (threadIdx.x + k * NTHR) / C::CPR;
        const int rr = row < nvalid ? row : nvalid - 1;
        if (SBASE) r.den[k] = *reinterpret_cast<const float *>(dbase + static_cast<uint32_t>(rr * 4));
        else r.den[k] = den[t0 + rr];
    }
}

template <class C, int ROWS, int STRIDE = C::XS, bool IL = false, int NTHR = kThreads>
__device__ __forceinline__ void store_cotangent(const CotChunks<C, ROWS, NTHR> &r, bf16raw *dst, float *ge, int L_real, int nvalid)
{
    const int tid = opaque(static_cast<int>(threadIdx.x));
#pragma unroll
    for (int k = 0; k < RowChunks<C, ROWS, NTHR>::N; ++k) {
        const int c = tid + k * NTHR, row = c / C::CPR, ch = c % C::CPR;
        // rows past the end of the tile hold a copy of the last real row: they get zero cotangents
        const float inv = (row < nvalid && r.den[k] > 0.f) ? __builtin_amdgcn_rcpf(r.den[k] * static_cast<float>(L_real)) : 0.f;
        const uint32_t gw[4] = {r.g.v[k].x, r.g.v[k].y, r.g.v[k].z, r.g.v[k].w};
        const uint32_t ow[4] = {r.o.v[k].x, r.o.v[k].y, r.o.v[k].z, r.o.v[k].w};
        uint32_t out[4];
        float dot = 0.f;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            out[e] = pack2(bf_lo(gw[e]) * inv, bf_hi(gw[e]) * inv);
            // the extra column is formed from the rounded cotangents the matrix products will see: for a row of the
            // statistics made of few keys, V_j . gn + ge = (V_j - O_i) . gn then cancels as it does in exact arithmetic
            dot = dot2(out[e], ow[e], dot);
        }
        if (row < ROWS) store_chunk<STRIDE, IL>(dst, row, ch, u32x4{out[0], out[1], out[2], out[3]});
        if (ge) {
            // the CPR threads of one row are consecutive lanes
#pragma unroll
            for (int m = C::CPR / 2; m >= 1; m >>= 1) dot += __shfl_xor(dot, m, 64);
            if (ch == 0 && row < ROWS) ge[row] = -dot;
        }
    }
}

// ---------------------------------------------------------------- projection + soft assignment
// z^T (32 projection rows of group g) x (32 tokens) = Wg . X^T, contraction over d (Algorithm 1, step 4:
// the argument of tanh).  Lane (n, h) ends up with the projections of token n for the TPL tables
// {g*TPG + h*TPL + j}: the host stores W's rows in that order (see pack_projection()).
// scale != null: the projections of token n are multiplied by scale[n] (W (x / |x|) = (W x) / |x|).
template <class C>
__device__ __forceinline__ f32x16 project(const bf16raw *wp, const bf16raw *x, int g, int ln, int h,
                                          const float *scale = nullptr)
{
    // two accumulators halve the chain of dependent MFMAs
    f32x16 z0 = {0}, z1 = {0};
#pragma unroll
    for (int s = 0; s < C::D / 16; s += 2) {
        z0 = mma(lds128(wp + (g * 32 + ln) * C::XS + 16 * s + 8 * h), lds128(x + ln * C::XS + 16 * s + 8 * h), z0);
        z1 = mma(lds128(wp + (g * 32 + ln) * C::XS + 16 * s + 16 + 8 * h), lds128(x + ln * C::XS + 16 * s + 16 + 8 * h), z1);
    }
    f32x16 z = z0 + z1;
    if (scale) z = z * scale[ln];
    return z;
}
// projection t of the lane's j-th table inside the accumulator
template <class C>
__device__ __forceinline__ constexpr int zslot(int j, int t)
{
    return C::PP == 8 ? 4 * (2 * j + t / 4) + t % 4 : 4 * j + t;
}

// Per-bit masses of one table: p[t] = sigmoid(2 beta tanh z_t) (mass on the +1 side), q[t] = 1 - p[t],
// computed without cancellation; sech2[t] = 1 - tanh^2 z_t; u[t] = tanh z_t.  Padding bits (t >= sf.P): all the
// mass on the +1 side, no dependence on the input.
template <class C>
__device__ __forceinline__ void bit_masses(const f32x16 &z, int j, const Soft &sf, float *p, float *q, float *sech2,
                                           float *u = nullptr)
{
    const float beta = sf.beta;
#pragma unroll
    for (int t = 0; t < C::P; ++t) {
        if (C::PAD && t >= sf.P) {
            p[t] = 1.f; q[t] = 0.f;
            if (sech2) sech2[t] = 0.f;
            if (u) u[t] = 0.f;
            continue;
        }
        const float zt = z[zslot<C>(j, t)];
        const float e2 = __expf(-2.0f * fabsf(zt));
        const float inv = __builtin_amdgcn_rcpf(1.0f + e2);
        const float ua = (1.0f - e2) * inv;                    // |tanh z|
        // beta = +infinity is the hard hash: e = 0, and at z = 0 (-inf * 0 = NaN; fmaxf returns its other argument) the bit is set
        const float e = __expf(fmaxf(-2.0f * beta * ua, -1e30f));
        const float big = __builtin_amdgcn_rcpf(1.0f + e), small = e * big;
        const bool pos = zt >= 0.f;
        p[t] = pos ? big : small;
        q[t] = pos ? small : big;
        if (sech2) sech2[t] = 4.0f * e2 * inv * inv;
        if (u) u[t] = pos ? ua : -ua;
    }
}

// The hashed form of one projection: c = +small or -small, where small = sigmoid(-2 beta |tanh z|) is the mass of the
// bit's minor side and the sign bit tells which side that is (clear: z >= 0, the major side is +1).  One float per
// (token, table, hyperplane) is all that the soft assignment of Algorithm 1, step 4 depends on: every pass after the
// first rebuilds phi from it instead of projecting and exponentiating again.  beta = +infinity gives +-0 (the hard
// hash); a padding hyperplane is +0 (all mass on the +1 side).
__device__ __forceinline__ float bit_code(float zt, float beta)
{
    const float e2 = __expf(-2.0f * fabsf(zt));
    const float ua = (1.0f - e2) * __builtin_amdgcn_rcpf(1.0f + e2);             // |tanh z|
    const float e = __expf(fmaxf(-2.0f * beta * ua, -1e30f));                    // (-inf * 0 = NaN at z = 0: fmaxf returns -1e30)
    const float small = e * __builtin_amdgcn_rcpf(1.0f + e);
    return zt >= 0.f ? small : -small;
}
// masses on the +1 side (p) and the -1 side (q) from the hashed form
__device__ __forceinline__ void code_masses(float c, float &p, float &q)
{
    const float small = fabsf(c), big = 1.0f - small;
    const bool pos = (__float_as_uint(c) >> 31) == 0;
    p = pos ? big : small;
    q = pos ? small : big;
}

// phi over the low PLO bits (lo) and the high PHI bits (hi): phi[a * 2^PLO + b] = hi[a] * lo[b]
// (the corner softmax is a product of per-bit two-point distributions).
template <class C>
__device__ __forceinline__ void kron_factors(const float *p, const float *q, float *lo, float *hi)
{
    lo[0] = 1.f;
#pragma unroll
    for (int t = 0; t < C::PLO; ++t) {
#pragma unroll
        for (int b = 0; b < (1 << t); ++b) {
            lo[b + (1 << t)] = lo[b] * p[t];
            lo[b] = lo[b] * q[t];
        }
    }
    hi[0] = 1.f;
#pragma unroll
    for (int t = 0; t < C::PHI; ++t) {
#pragma unroll
        for (int b = 0; b < (1 << t); ++b) {
            hi[b + (1 << t)] = hi[b] * p[C::PLO + t];
            hi[b] = hi[b] * q[C::PLO + t];
        }
    }
}

// Writes the assignment of the lane's token as bf16 into row `row` of ph [token][L*R] (row stride STRIDE),
// corners pair-interleaved: the 16 corners of high-bit indices (a, a+1), a even, are stored as
// [a: b 0..3 | a+1: b 0..3 | a: b 4..7 | a+1: b 4..7].
// valid == false writes zeros (a token past the end of the sequence must not reach the statistics).
// Only the lane's tables j = j0, j0 + jstep, ... and the high-bit indices a0 <= a < a1 (both even) are
// written, which lets several wavefronts share the tables of one projection group.
// If mass != null (bucket masses in the same pair-interleaved order), returns sum_r phi[r] * mass[r] over
// what was written (the read-out of the bucket masses A by this token, i.e. its share of the normaliser).
// Two sources: the projections z of the lane's token (an accumulator of project()), or, if mrow != null, the hashed
// row of the lane's token (C::LP floats, see bit_code()).
// FENCE: a scheduling fence after every pair of high-bit indices (bounds the registers the compiler may spend on
// interleaving them; kernels with registers to spare turn it off).
template <class C, int STRIDE = C::PS, bool FENCE = true>
__device__ __forceinline__ float write_assignments(const f32x16 &z, int g, int row, int h, const Soft &sf, bool valid,
                                                   bf16raw *ph, int j0 = 0, int jstep = 1, int a0 = 0,
                                                   int a1 = 1 << C::PHI, const float *mass = nullptr,
                                                   const float *mrow = nullptr)
{
    static_assert(C::PLO == 3 && C::PHI >= 1, "eight low corners per high-bit index, indices in pairs");
    float dn = 0.f;
#pragma unroll
    for (int j = 0; j < C::TPL; ++j) {
        const int table = g * C::TPG + h * C::TPL + j;
        if (table >= C::L) break;
        if (j < j0 || (j - j0) % jstep != 0) continue;
        const int tbase = opaque(table * C::R);                   // one base register, constants folded into offsets
        bf16raw *prow = ph + opaque(row * STRIDE);
        if (C::PAD && table >= sf.L) {                            // a padding table: zero assignments
#pragma unroll
            for (int a = 0; a < (1 << C::PHI); a += 2) {
                if (a < a0 || a >= a1) continue;
                *reinterpret_cast<u32x4 *>(prow + tbase + a * 8) = u32x4{0u, 0u, 0u, 0u};
                *reinterpret_cast<u32x4 *>(prow + tbase + a * 8 + 8) = u32x4{0u, 0u, 0u, 0u};
            }
            continue;
        }
        float p[C::P], q[C::P], lo[1 << C::PLO], hi[1 << C::PHI];
        if (mrow) {
            const float *src = mrow + opaque(table * C::P);
#pragma unroll
            for (int t = 0; t < C::P; t += 2) {
                const float2 c2 = *reinterpret_cast<const float2 *>(src + t);
                code_masses(c2.x, p[t], q[t]);
                code_masses(c2.y, p[t + 1], q[t + 1]);
            }
        } else {
            bit_masses<C>(z, j, sf, p, q, nullptr);
        }
        kron_factors<C>(p, q, lo, hi);
#pragma unroll
        for (int a = 0; a < (1 << C::PHI); a += 2) {
            if (a < a0 || a >= a1) continue;
            const float ha = valid ? hi[a] : 0.f, hb = valid ? hi[a + 1] : 0.f;
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                const int pos = tbase + a * 8 + 8 * half;
                float f[8];
#pragma unroll
                for (int b = 0; b < 4; ++b) { f[b] = ha * lo[4 * half + b]; f[4 + b] = hb * lo[4 * half + b]; }
                if (mass) {
                    const float4 m0 = *reinterpret_cast<const float4 *>(mass + pos);
                    const float4 m1 = *reinterpret_cast<const float4 *>(mass + pos + 4);
                    dn = fmaf(f[0], m0.x, dn); dn = fmaf(f[1], m0.y, dn); dn = fmaf(f[2], m0.z, dn); dn = fmaf(f[3], m0.w, dn);
                    dn = fmaf(f[4], m1.x, dn); dn = fmaf(f[5], m1.y, dn); dn = fmaf(f[6], m1.z, dn); dn = fmaf(f[7], m1.w, dn);
                }
                *reinterpret_cast<u32x4 *>(prow + pos) =
                    u32x4{pack2(f[0], f[1]), pack2(f[2], f[3]), pack2(f[4], f[5]), pack2(f[6], f[7])};
            }
            if (FENCE) RACE_SCHED_FENCE();
        }
    }
    return dn;
}

}  // namespace mfma
}  // namespace race
