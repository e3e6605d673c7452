// Generic RACE Attention kernels: any (L, P <= 8, d <= 256), fp32 or bf16 tensors, all arithmetic
// in fp32 on the vector ALUs.  One workgroup owns one (batch*head, table, segment): the table's
// bucket statistics [R][d+1] (B | A of Algorithm 1, step 5) live in LDS and tokens are taken in
// the order of Algorithm 2 (update with key/value t, then query t reads).  Per-table partial
// numerators are written to the workspace and summed over tables in table order by a combine
// kernel, so results are deterministic.  This family serves the fp32 element type and every bf16
// shape the MFMA family has no instantiation for; it is written for clarity, not speed.
#include <hip/hip_runtime.h>

#include "internal.h"

namespace race {
namespace {

constexpr int kThreads = 256;

// ------------------------------------------------------------------ element access
struct bf16_t { uint16_t bits; };

__device__ __forceinline__ float load_elem(const float *p, size_t i) { return p[i]; }
__device__ __forceinline__ float load_elem(const bf16_t *p, size_t i)
{
    return __uint_as_float(static_cast<uint32_t>(p[i].bits) << 16);
}
__device__ __forceinline__ void store_elem(float *p, size_t i, float v) { p[i] = v; }
__device__ __forceinline__ void store_elem(bf16_t *p, size_t i, float v)
{
    uint32_t b = __float_as_uint(v);
    if ((b & 0x7fffffffu) > 0x7f800000u) { p[i].bits = 0x7fc0; return; }      // NaN
    b += 0x7fffu + ((b >> 16) & 1u);                                          // nearest even
    p[i].bits = static_cast<uint16_t>(b >> 16);
}

struct Args {
    int H, L, P, R, d, LP, nseg, causal, TT;
    int unit;            // 1: rows of Q and K are divided by their Euclidean norms before the projection
    int64_t N, seg_len;
    float beta;
    const float *W;      // (H, L*P, d)
};

// ------------------------------------------------------------------ LDS carving
// S     [R][d+1]   bucket statistics of this table (value sums | mass)
// xa,xb [TT][d]    rows of the two hashed tensors
// ya,yb [TT][d+1]  rows of the two accumulated tensors ([V | 1] and [dO/e | -(dO.O)/e])
// ha,hb            per-token hash data of the two hashed tensors: s, p, q, u, z [TT][P] each, phi [TT][R], inv [TT]
// dphi  [R], dz [P]
struct Smem {
    float *S, *xa, *xb, *ya, *yb, *ha, *hb, *dphi, *dz;
    __device__ Smem(float *base, const Args &a)
    {
        const int d1 = a.d + 1;
        S = base;                 base += a.R * d1;
        xa = base;                base += a.TT * a.d;
        xb = base;                base += a.TT * a.d;
        ya = base;                base += a.TT * d1;
        yb = base;                base += a.TT * d1;
        ha = base;                base += a.TT * (5 * a.P + a.R + 1);
        hb = base;                base += a.TT * (5 * a.P + a.R + 1);
        dphi = base;              base += a.R;
        dz = base;
    }
};
inline size_t smem_floats(int R, int d, int P, int TT)
{
    return static_cast<size_t>(R) * (d + 1) + 2 * TT * d + 2 * TT * (d + 1) + 2 * TT * (5 * P + R + 1) + R + P;
}

struct HashView {
    float *s, *p, *q, *u, *z, *phi; // s = 1 - tanh^2(z), p/q = mass on the +1/-1 side of each bit, u = tanh z
    float *inv;                     // 1 / max(|x|, floor) of the row (unit-norm option), else 1
    __device__ HashView(float *h, const Args &a)
        : s(h), p(h + a.TT * a.P), q(h + 2 * a.TT * a.P), u(h + 3 * a.TT * a.P), z(h + 4 * a.TT * a.P),
          phi(h + 5 * a.TT * a.P), inv(h + 5 * a.TT * a.P + a.TT * a.R) {}
};

// rows [t0, t0+nt) of X -> xs[TT][d]
template <typename T>
__device__ void load_rows(const T *X, size_t row0, int nt, int d, float *xs)
{
    for (int i = threadIdx.x; i < nt * d; i += kThreads) xs[i] = load_elem(X, row0 * d + i);
}

// [V | 1] rows
template <typename T>
__device__ void load_value_rows(const T *V, size_t row0, int nt, int d, float *ys)
{
    for (int i = threadIdx.x; i < nt * (d + 1); i += kThreads) {
        const int t = i / (d + 1), c = i - t * (d + 1);
        ys[i] = (c < d) ? load_elem(V, (row0 + t) * d + c) : 1.0f;
    }
}

// [dO / e | -(dO . O) / e] rows with e = L * Den: the cotangents of the un-averaged numerator and
// normaliser of Algorithm 1, step 7.  scratch: [TT][d] floats.
template <typename T>
__device__ void load_cotangent_rows(const T *dO, const T *O, const float *den, size_t row0, int nt, int d,
                                    int L, float *ys, float *scratch)
{
    for (int i = threadIdx.x; i < nt * d; i += kThreads) {
        const int t = i / d, c = i - t * d;
        const float g = load_elem(dO, (row0 + t) * d + c);
        ys[t * (d + 1) + c] = g;
        scratch[i] = g * load_elem(O, (row0 + t) * d + c);
    }
    __syncthreads();
    // 32 threads per token
    const int t = threadIdx.x >> 5, sub = threadIdx.x & 31;
    for (int tok = t; tok < nt; tok += kThreads / 32) {
        float acc = 0.f;
        for (int c = sub; c < d; c += 32) acc += scratch[tok * d + c];
        for (int m = 16; m >= 1; m >>= 1) acc += __shfl_xor(acc, m, 64);
        const float inv = 1.0f / (den[row0 + tok] * static_cast<float>(L));
        for (int c = sub; c < d; c += 32) ys[tok * (d + 1) + c] *= inv;
        if (sub == 0) ys[tok * (d + 1) + d] = -acc * inv;
    }
    __syncthreads();
}

// Projection + soft assignment of nt rows (Algorithm 1, steps 2-4).  phi is built from its
// factorised form phi_r = prod_t sigmoid(2 beta v_{r,t} u_t), u = tanh(W x), which equals the
// e = exp(-2 beta |u|), the ratio of the two masses of a bit.  beta = +infinity is the hard hash of Section 3.3:
// e = 0 for u != 0, and for u = 0 (where -inf * 0 is NaN; fmaxf returns its other argument) the bit counts as set, like z >= 0.
__device__ __forceinline__ float mass_ratio(float beta, float u)
{
    return expf(fmaxf(-2.0f * beta * fabsf(u), -1e30f));
}

// Unit-norm option (the setting of Theorem 1's proof, |Q_i| = |K_j| = 1): the factor that turns a row of squared
// length ss into a unit vector; rows shorter than the floor are divided by the floor (a zero row stays zero).
constexpr float kUnitFloor = 1e-12f;
__device__ __forceinline__ float unit_scale(float ss) { return 1.0f / fmaxf(sqrtf(ss), kUnitFloor); }

// softmax over corners exactly (the softmax denominator is prod_t 2 cosh(beta u_t)).
__device__ void hash_rows(const Args &a, const float *Wl, const float *xs, int nt, HashView hv)
{
    __syncthreads();
    const int sub = threadIdx.x & 3;
    for (int pair = threadIdx.x >> 2; pair < nt * a.P; pair += kThreads / 4) {
        const int tok = pair / a.P, t = pair - tok * a.P;
        float z = 0.f, ss = 0.f;
        for (int c = sub; c < a.d; c += 4) {
            const float x = xs[tok * a.d + c];
            z = fmaf(Wl[t * a.d + c], x, z);
            ss = fmaf(x, x, ss);
        }
        z += __shfl_xor(z, 1, 64);
        z += __shfl_xor(z, 2, 64);
        ss += __shfl_xor(ss, 1, 64);
        ss += __shfl_xor(ss, 2, 64);
        if (sub == 0) {
            const float inv = a.unit ? unit_scale(ss) : 1.0f;
            z *= inv;                                              // W (x / |x|)
            if (t == 0) hv.inv[tok] = inv;
            hv.z[pair] = z;
            const float u = tanhf(z);
            const float e = mass_ratio(a.beta, u);                  // in [0, 1]
            const float big = 1.0f / (1.0f + e), small = e / (1.0f + e);
            const float e2 = expf(-2.0f * fabsf(z));               // 1 - tanh^2 z = 4 e2 / (1 + e2)^2
            hv.u[pair] = u;
            hv.s[pair] = 4.0f * e2 / ((1.0f + e2) * (1.0f + e2));
            hv.p[pair] = (u >= 0.f) ? big : small;                 // mass on the +1 side of bit t
            hv.q[pair] = (u >= 0.f) ? small : big;
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < nt * a.R; i += kThreads) {
        const int tok = i / a.R, r = i - tok * a.R;
        float f = 1.f;
        for (int t = 0; t < a.P; ++t) f *= ((r >> t) & 1) ? hv.p[tok * a.P + t] : hv.q[tok * a.P + t];
        hv.phi[i] = f;
    }
    __syncthreads();
}

// S[:, c] += phi[r] * y[c] for the columns this thread owns (thread-private columns: no barrier).
__device__ __forceinline__ void accumulate_token(const Args &a, float *S, const float *phi, const float *y)
{
    const int d1 = a.d + 1;
    for (int c = threadIdx.x; c < d1; c += kThreads) {
        const float yc = y[c];
        for (int r = 0; r < a.R; ++r) S[r * d1 + c] = fmaf(phi[r], yc, S[r * d1 + c]);
    }
}

// Cotangent of phi -> cotangent of z (softmax over corners, corner logits, tanh).  dphi in LDS.
// Leaves dz[P] in LDS (followed by a barrier).  Thread t < P also adds its bit's share of the cotangent of
// beta, du_t * u_t (the corner logits are beta * (u . v_r)), to dbeta_acc.
__device__ void soft_hash_vjp(const Args &a, const float *phi, const float *sech2, const float *u, const float *dphi,
                              float *dz, float &dbeta_acc)
{
    if (threadIdx.x < a.P) {
        const int t = threadIdx.x;
        float mean = 0.f;
        for (int r = 0; r < a.R; ++r) mean = fmaf(phi[r], dphi[r], mean);
        float du = 0.f;
        for (int r = 0; r < a.R; ++r) {
            const float ds = phi[r] * (dphi[r] - mean);
            du += ((r >> t) & 1) ? ds : -ds;
        }
        dz[t] = a.beta * du * sech2[t];
        dbeta_acc = fmaf(du, u[t], dbeta_acc);
    }
    __syncthreads();
}

// Chain rule through x -> x / |x| for one token and table: with g = W^T dz the cotangent of the unit vector,
// dx = (g - xhat (xhat . g)) / |x|, and xhat . g = z . dz because z = W xhat.  Returns (1 / |x|, (z . dz) / |x|^2):
// dx = .x * g - .y * x.  Without the option: (1, 0).
__device__ __forceinline__ float2 unit_terms(const Args &a, const HashView &hv, int tok, const float *dz)
{
    if (!a.unit) return float2{1.f, 0.f};
    const float inv = hv.inv[tok];
    float radial = 0.f;
    for (int t = 0; t < a.P; ++t) radial = fmaf(hv.z[tok * a.P + t], dz[t], radial);
    return float2{inv, radial * inv * inv};
}

// Sum of the first P threads' dbeta_acc, in thread order, to one workspace slot (end of a gradient kernel).
__device__ void store_dbeta_partial(const Args &a, float dbeta_acc, float *scratch, float *slot)
{
    __syncthreads();
    if (threadIdx.x < a.P) scratch[threadIdx.x] = dbeta_acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        float s = 0.f;
        for (int t = 0; t < a.P; ++t) s += scratch[t];
        *slot = s;
    }
}

__device__ __forceinline__ size_t state_index(const Args &a, int bh, int l, int seg)
{
    return ((static_cast<size_t>(bh) * a.L + l) * a.nseg + seg) * a.R * (a.d + 1);
}

// ------------------------------------------------------------------ kernels
// Segment totals of the bucket statistics.  SIDE 0: keys/values (A | B of Algorithm 1, step 5).
// SIDE 1: queries / read-out cotangents (the statistics the key side reads in the backward pass).
template <typename T, int SIDE>
__global__ __launch_bounds__(kThreads) void simple_totals(Args a, const T *X, const T *Y, const T *O,
                                                          const float *den, float *state)
{
    extern __shared__ float lds[];
    Smem sm(lds, a);
    const int seg = blockIdx.x, l = blockIdx.y, bh = blockIdx.z, h = bh % a.H;
    const float *Wl = a.W + (static_cast<size_t>(h) * a.LP + l * a.P) * a.d;
    const int d1 = a.d + 1;
    for (int i = threadIdx.x; i < a.R * d1; i += kThreads) sm.S[i] = 0.f;
    const int64_t t_begin = seg * a.seg_len;
    const int64_t t_end = (t_begin + a.seg_len < a.N) ? t_begin + a.seg_len : a.N;
    HashView hv(sm.ha, a);
    for (int64_t t0 = t_begin; t0 < t_end; t0 += a.TT) {
        const int nt = (t_end - t0 < a.TT) ? static_cast<int>(t_end - t0) : a.TT;
        const size_t row0 = static_cast<size_t>(bh) * a.N + t0;
        __syncthreads();
        load_rows(X, row0, nt, a.d, sm.xa);
        if (SIDE == 0) load_value_rows(Y, row0, nt, a.d, sm.ya);
        else load_cotangent_rows(Y, O, den, row0, nt, a.d, a.L, sm.ya, sm.xb);
        hash_rows(a, Wl, sm.xa, nt, hv);
        for (int tok = 0; tok < nt; ++tok) accumulate_token(a, sm.S, hv.phi + tok * a.R, sm.ya + tok * d1);
    }
    __syncthreads();
    float *out = state + state_index(a, bh, l, seg);
    for (int i = threadIdx.x; i < a.R * d1; i += kThreads) out[i] = sm.S[i];
}

// In-place scan over segments of the per-segment totals.  mode 0: exclusive prefix (state at the
// start of the segment, forward direction); 1: exclusive suffix; 2: every segment gets the grand total.
__global__ void simple_scan(float *state, int nseg, size_t elems, int mode)
{
    const size_t e = blockIdx.x * static_cast<size_t>(blockDim.x) + threadIdx.x;
    if (e >= elems) return;
    float *base = state + static_cast<size_t>(blockIdx.y) * nseg * elems + e;
    if (mode == 0) {
        float run = 0.f;
        for (int s = 0; s < nseg; ++s) { const float v = base[s * elems]; base[s * elems] = run; run += v; }
    } else if (mode == 1) {
        float run = 0.f;
        for (int s = nseg - 1; s >= 0; --s) { const float v = base[s * elems]; base[s * elems] = run; run += v; }
    } else {
        float run = 0.f;
        for (int s = 0; s < nseg; ++s) run += base[s * elems];
        for (int s = 0; s < nseg; ++s) base[s * elems] = run;
    }
}

// Forward replay of one segment of one table: Algorithm 2's loop body (or Algorithm 1's read-out
// against the all-N statistics).  Writes the table's un-averaged [num | den] rows.
template <typename T>
__global__ __launch_bounds__(kThreads) void simple_fwd_replay(Args a, const T *Q, const T *K, const T *V,
                                                              const float *state, float *part)
{
    extern __shared__ float lds[];
    Smem sm(lds, a);
    const int seg = blockIdx.x, l = blockIdx.y, bh = blockIdx.z, h = bh % a.H;
    const float *Wl = a.W + (static_cast<size_t>(h) * a.LP + l * a.P) * a.d;
    const int d1 = a.d + 1;
    const float *init = state + state_index(a, bh, l, seg);
    for (int i = threadIdx.x; i < a.R * d1; i += kThreads) sm.S[i] = init[i];
    const int64_t t_begin = seg * a.seg_len;
    const int64_t t_end = (t_begin + a.seg_len < a.N) ? t_begin + a.seg_len : a.N;
    HashView hk(sm.ha, a), hq(sm.hb, a);
    float *out = part + (static_cast<size_t>(bh) * a.L + l) * a.N * d1;
    for (int64_t t0 = t_begin; t0 < t_end; t0 += a.TT) {
        const int nt = (t_end - t0 < a.TT) ? static_cast<int>(t_end - t0) : a.TT;
        const size_t row0 = static_cast<size_t>(bh) * a.N + t0;
        __syncthreads();
        load_rows(Q, row0, nt, a.d, sm.xb);
        if (a.causal) {
            load_rows(K, row0, nt, a.d, sm.xa);
            load_value_rows(V, row0, nt, a.d, sm.ya);
            hash_rows(a, Wl, sm.xa, nt, hk);
        }
        hash_rows(a, Wl, sm.xb, nt, hq);
        for (int tok = 0; tok < nt; ++tok) {
            if (a.causal) accumulate_token(a, sm.S, hk.phi + tok * a.R, sm.ya + tok * d1);
            const float *phi = hq.phi + tok * a.R;
            for (int c = threadIdx.x; c < d1; c += kThreads) {
                float acc = 0.f;
                for (int r = 0; r < a.R; ++r) acc = fmaf(phi[r], sm.S[r * d1 + c], acc);
                out[(t0 + tok) * d1 + c] = acc;
            }
        }
    }
}

// Num = (1/L) sum_l num_l, Den = (1/L) sum_l den_l, O = Num / Den  (Algorithm 1, steps 7-8)
template <typename T>
__global__ void simple_fwd_combine(Args a, int BH, const float *part, T *O, float *den)
{
    const size_t i = blockIdx.x * static_cast<size_t>(blockDim.x) + threadIdx.x;
    const size_t total = static_cast<size_t>(BH) * a.N * a.d;
    if (i >= total) return;
    const int d1 = a.d + 1;
    const size_t row = i / a.d;
    const int c = static_cast<int>(i - row * a.d);
    const size_t bh = row / a.N, t = row - bh * a.N;
    float num = 0.f, dn = 0.f;
    for (int l = 0; l < a.L; ++l) {
        const float *p = part + ((bh * a.L + l) * a.N + t) * d1;
        num += p[c];
        dn += p[a.d];
    }
    const float invL = 1.0f / static_cast<float>(a.L);
    store_elem(O, i, dn > 0.f ? (num * invL) / (dn * invL) : 0.f);      // dn = 0: only the hard hash, empty buckets
    if (c == 0) den[row] = dn * invL;
}

// Backward, query side, one segment of one table, left to right: with the prefix statistics S
// (after adding key/value i), dphi_Q[r] = S[r,:] . [dO_i/e_i | -(dO_i.O_i)/e_i]; then back through
// the soft assignment to the table's share of dQ_i.
template <typename T>
__global__ __launch_bounds__(kThreads) void simple_bwd_query(Args a, const T *Q, const T *K, const T *V,
                                                             const T *O, const float *den, const T *dO,
                                                             const float *state, float *partQ, float *dbeta_part)
{
    extern __shared__ float lds[];
    Smem sm(lds, a);
    const int seg = blockIdx.x, l = blockIdx.y, bh = blockIdx.z, h = bh % a.H;
    const float *Wl = a.W + (static_cast<size_t>(h) * a.LP + l * a.P) * a.d;
    const int d1 = a.d + 1;
    const float *init = state + state_index(a, bh, l, seg);
    for (int i = threadIdx.x; i < a.R * d1; i += kThreads) sm.S[i] = init[i];
    const int64_t t_begin = seg * a.seg_len;
    const int64_t t_end = (t_begin + a.seg_len < a.N) ? t_begin + a.seg_len : a.N;
    HashView hk(sm.ha, a), hq(sm.hb, a);
    float dbeta_acc = 0.f;          // threads t < P: this workgroup's share of the cotangent of beta, bit t
    float *out = partQ + (static_cast<size_t>(bh) * a.L + l) * a.N * a.d;
    for (int64_t t0 = t_begin; t0 < t_end; t0 += a.TT) {
        const int nt = (t_end - t0 < a.TT) ? static_cast<int>(t_end - t0) : a.TT;
        const size_t row0 = static_cast<size_t>(bh) * a.N + t0;
        __syncthreads();
        if (a.causal) {
            load_rows(K, row0, nt, a.d, sm.xa);
            load_value_rows(V, row0, nt, a.d, sm.ya);
            hash_rows(a, Wl, sm.xa, nt, hk);
        }
        load_cotangent_rows(dO, O, den, row0, nt, a.d, a.L, sm.yb, sm.xb);
        load_rows(Q, row0, nt, a.d, sm.xb);
        hash_rows(a, Wl, sm.xb, nt, hq);
        for (int tok = 0; tok < nt; ++tok) {
            if (a.causal) {
                accumulate_token(a, sm.S, hk.phi + tok * a.R, sm.ya + tok * d1);
                __syncthreads();
            }
            const float *gt = sm.yb + tok * d1;
            for (int r = threadIdx.x; r < a.R; r += kThreads) {
                float acc = 0.f;
                for (int c = 0; c < d1; ++c) acc = fmaf(sm.S[r * d1 + c], gt[c], acc);
                sm.dphi[r] = acc;
            }
            __syncthreads();
            soft_hash_vjp(a, hq.phi + tok * a.R, hq.s + tok * a.P, hq.u + tok * a.P, sm.dphi, sm.dz, dbeta_acc);
            const float2 un = unit_terms(a, hq, tok, sm.dz);
            for (int c = threadIdx.x; c < a.d; c += kThreads) {
                float acc = 0.f;
                for (int t = 0; t < a.P; ++t) acc = fmaf(sm.dz[t], Wl[t * a.d + c], acc);
                out[(t0 + tok) * a.d + c] = un.x * acc - un.y * sm.xb[tok * a.d + c];
            }
            __syncthreads();
        }
    }
    // side 0 (queries) of the (2, BH, L * nseg) partial cotangents of beta
    store_dbeta_partial(a, dbeta_acc, sm.dphi, dbeta_part + (static_cast<size_t>(bh) * a.L + l) * a.nseg + seg);
}

// Backward, key/value side, one segment of one table, right to left: with the suffix statistics
// dS of the read-out cotangents (after adding query j), dV_j = phi_K(j) . dB,
// dphi_K[r] = dB[r,:] . V_j + dA[r]; then back through the soft assignment to the share of dK_j.
template <typename T>
__global__ __launch_bounds__(kThreads) void simple_bwd_keyvalue(Args a, const T *Q, const T *K, const T *V,
                                                                const T *O, const float *den, const T *dO,
                                                                const float *state, float *partK, float *partV,
                                                                float *dbeta_part)
{
    extern __shared__ float lds[];
    Smem sm(lds, a);
    const int seg = blockIdx.x, l = blockIdx.y, bh = blockIdx.z, h = bh % a.H;
    const float *Wl = a.W + (static_cast<size_t>(h) * a.LP + l * a.P) * a.d;
    const int d1 = a.d + 1;
    const float *init = state + state_index(a, bh, l, seg);
    for (int i = threadIdx.x; i < a.R * d1; i += kThreads) sm.S[i] = init[i];
    const int64_t t_begin = seg * a.seg_len;
    const int64_t t_end = (t_begin + a.seg_len < a.N) ? t_begin + a.seg_len : a.N;
    HashView hk(sm.ha, a), hq(sm.hb, a);
    float dbeta_acc = 0.f;          // threads t < P: this workgroup's share of the cotangent of beta, bit t
    float *outK = partK + (static_cast<size_t>(bh) * a.L + l) * a.N * a.d;
    float *outV = partV + (static_cast<size_t>(bh) * a.L + l) * a.N * a.d;
    const int64_t ntiles = (t_end - t_begin + a.TT - 1) / a.TT;
    for (int64_t tile = ntiles - 1; tile >= 0; --tile) {
        const int64_t t0 = t_begin + tile * a.TT;
        const int nt = (t_end - t0 < a.TT) ? static_cast<int>(t_end - t0) : a.TT;
        const size_t row0 = static_cast<size_t>(bh) * a.N + t0;
        __syncthreads();
        load_rows(K, row0, nt, a.d, sm.xa);
        load_value_rows(V, row0, nt, a.d, sm.ya);
        hash_rows(a, Wl, sm.xa, nt, hk);
        if (a.causal) {
            load_cotangent_rows(dO, O, den, row0, nt, a.d, a.L, sm.yb, sm.xb);
            load_rows(Q, row0, nt, a.d, sm.xb);
            hash_rows(a, Wl, sm.xb, nt, hq);
        }
        for (int tok = nt - 1; tok >= 0; --tok) {
            if (a.causal) accumulate_token(a, sm.S, hq.phi + tok * a.R, sm.yb + tok * d1);
            const float *phi = hk.phi + tok * a.R;
            for (int c = threadIdx.x; c < a.d; c += kThreads) {       // same columns as accumulate_token
                float acc = 0.f;
                for (int r = 0; r < a.R; ++r) acc = fmaf(phi[r], sm.S[r * d1 + c], acc);
                outV[(t0 + tok) * a.d + c] = acc;
            }
            __syncthreads();
            const float *vt = sm.ya + tok * d1;
            for (int r = threadIdx.x; r < a.R; r += kThreads) {
                float acc = 0.f;
                for (int c = 0; c < d1; ++c) acc = fmaf(sm.S[r * d1 + c], vt[c], acc);
                sm.dphi[r] = acc;
            }
            __syncthreads();
            soft_hash_vjp(a, phi, hk.s + tok * a.P, hk.u + tok * a.P, sm.dphi, sm.dz, dbeta_acc);
            const float2 un = unit_terms(a, hk, tok, sm.dz);
            for (int c = threadIdx.x; c < a.d; c += kThreads) {
                float acc = 0.f;
                for (int t = 0; t < a.P; ++t) acc = fmaf(sm.dz[t], Wl[t * a.d + c], acc);
                outK[(t0 + tok) * a.d + c] = un.x * acc - un.y * sm.xa[tok * a.d + c];
            }
            __syncthreads();
        }
    }
    // side 1 (keys)
    store_dbeta_partial(a, dbeta_acc, sm.dphi,
                        dbeta_part + ((static_cast<size_t>(gridDim.z) + bh) * a.L + l) * a.nseg + seg);
}

template <typename T>
__global__ void simple_bwd_combine(Args a, int BH, const float *pQ, const float *pK, const float *pV,
                                   T *dQ, T *dK, T *dV)
{
    const size_t i = blockIdx.x * static_cast<size_t>(blockDim.x) + threadIdx.x;
    const size_t total = static_cast<size_t>(BH) * a.N * a.d;
    if (i >= total) return;
    const size_t row = i / a.d;
    const int c = static_cast<int>(i - row * a.d);
    const size_t bh = row / a.N, t = row - bh * a.N;
    float q = 0.f, k = 0.f, v = 0.f;
    for (int l = 0; l < a.L; ++l) {
        const size_t j = ((bh * a.L + l) * a.N + t) * a.d + c;
        q += pQ[j]; k += pK[j]; v += pV[j];
    }
    store_elem(dQ, i, q);
    store_elem(dK, i, k);
    store_elem(dV, i, v);
}

// Debug tap: hard codes and phi of every (row, table).
template <typename T>
__global__ void simple_hash_tap(Args a, int BH, const T *X, uint8_t *codes, float *phi)
{
    const size_t i = blockIdx.x * static_cast<size_t>(blockDim.x) + threadIdx.x;
    const size_t total = static_cast<size_t>(BH) * a.N * a.L;
    if (i >= total) return;
    const size_t row = i / a.L;
    const int l = static_cast<int>(i - row * a.L);
    const int h = static_cast<int>((row / a.N) % a.H);
    const float *Wl = a.W + (static_cast<size_t>(h) * a.LP + l * a.P) * a.d;
    float p[8], q[8];
    unsigned code = 0;
    float inv = 1.f;
    if (a.unit) {
        float ss = 0.f;
        for (int c = 0; c < a.d; ++c) { const float x = load_elem(X, row * a.d + c); ss = fmaf(x, x, ss); }
        inv = unit_scale(ss);
    }
    for (int t = 0; t < a.P; ++t) {
        float z = 0.f;
        for (int c = 0; c < a.d; ++c) z = fmaf(Wl[t * a.d + c], load_elem(X, row * a.d + c), z);
        z *= inv;
        code |= (z >= 0.f ? 1u : 0u) << t;
        const float u = tanhf(z);
        const float e = mass_ratio(a.beta, u);
        const float big = 1.0f / (1.0f + e), small = e / (1.0f + e);
        p[t] = (u >= 0.f) ? big : small;
        q[t] = (u >= 0.f) ? small : big;
    }
    codes[i] = static_cast<uint8_t>(code);
    if (phi) {
        for (int r = 0; r < a.R; ++r) {
            float f = 1.f;
            for (int t = 0; t < a.P; ++t) f *= ((r >> t) & 1) ? p[t] : q[t];
            phi[i * a.R + r] = f;
        }
    }
}

// Sum of the per-segment totals, written as A[row * a_stride] and Bsum[row * b_stride + c], row = (bh, l, r).
__global__ void simple_bucket_tap(Args a, int BH, const float *state, float *A, float *Bsum, int a_stride, int b_stride)
{
    const size_t i = blockIdx.x * static_cast<size_t>(blockDim.x) + threadIdx.x;
    const int d1 = a.d + 1;
    const size_t total = static_cast<size_t>(BH) * a.L * a.R * d1;
    if (i >= total) return;
    const size_t bl = i / (static_cast<size_t>(a.R) * d1);
    const size_t e = i - bl * a.R * d1;
    float run = 0.f;
    for (int s = 0; s < a.nseg; ++s) run += state[(bl * a.nseg + s) * a.R * d1 + e];
    const int r = static_cast<int>(e / d1), c = static_cast<int>(e - static_cast<size_t>(r) * d1);
    if (c == a.d) A[(bl * a.R + r) * a_stride] = run;
    else Bsum[(bl * a.R + r) * b_stride + c] = run;
}

// ------------------------------------------------------------------ incremental decoding
// One decoding step, one workgroup of 1024 threads per (batch, head).  Threads form TF = 1024 / TL slots of
// TL = 64 ceil(d / 64) threads; a slot takes the tables slot, slot + TF, ... one after the other, thread c of a slot
// owning column c: it hashes the new key and query against the table's hyperplanes with its slot-mates (Algorithm 1,
// steps 2-4), adds the key/value to the table's statistics and reads them with the query, column by column
// (Algorithm 2's loop body; coalesced rows of d+1 floats).  The sums over tables and the normalisation follow in the
// same kernel (Algorithm 1, steps 7-8): numerators over the slots in slot order, the normaliser over the wavefronts.
constexpr int kDecodeThreads = 1024;

template <typename T>
__global__ __launch_bounds__(kDecodeThreads) void decode_step_kernel(int H, int L, int P, int d, float beta, int unit, const float *W,
                                                                     const T *q, const T *k, const T *v, float *state,
                                                                     T *o, float *den)
{
    extern __shared__ float lds[];
    const int R = 1 << P, d1 = d + 1;
    const int TL = (d + 63) & ~63, TF = kDecodeThreads / TL, NWV = TL / 64;
    const int tid = threadIdx.x, slot = tid / TL, c = tid % TL, lane = tid & 63, wv = c >> 6;
    const int bh = blockIdx.x, h = bh % H;
    float *zred = lds;                              // [TF][2P+2][NWV] partial projections, then the rows' squared lengths
    float *pq = zred + TF * (2 * P + 2) * NWV;      // [TF][2P][2]   per-bit masses (+1 side, -1 side)
    float *phi = pq + TF * 2 * P * 2;               // [TF][2][R]    assignments of the query (0) and the key (1)
    float *numred = phi + TF * 2 * R;               // [TF][d]       numerators per slot
    float *dred = numred + TF * d;                  // [16]          normaliser per wavefront
    const bool active = slot < TF, colok = active && c < d;
    const float xq = colok ? load_elem(q, static_cast<size_t>(bh) * d + c) : 0.f;
    const float xk = colok ? load_elem(k, static_cast<size_t>(bh) * d + c) : 0.f;
    const float vv = colok ? load_elem(v, static_cast<size_t>(bh) * d + c) : 0.f;
    float num = 0.f, dn = 0.f;
    for (int l0 = 0; l0 < L; l0 += TF) {
        const int l = l0 + slot;
        const bool on = active && l < L;
        const float *Wl = W + (static_cast<size_t>(h) * L + (on ? l : 0)) * P * d;
        for (int t = 0; t <= P; ++t) {              // t = P: the squared lengths |q|^2, |k|^2 instead of a projection
            const float w = (on && c < d) ? (t < P ? Wl[t * d + c] : 1.f) : 0.f;
            float a = w * xq * (t < P ? 1.f : xq), b = w * xk * (t < P ? 1.f : xk);
#pragma unroll
            for (int m = 32; m >= 1; m >>= 1) {
                a += __shfl_xor(a, m, 64);
                b += __shfl_xor(b, m, 64);
            }
            if (active && lane == 0) {
                zred[(slot * (2 * P + 2) + 2 * t) * NWV + wv] = a;
                zred[(slot * (2 * P + 2) + 2 * t + 1) * NWV + wv] = b;
            }
        }
        __syncthreads();
        if (on && c < 2 * P) {                      // per-bit masses of the query (c < P) and of the key
            const int side = c / P, t = c % P;
            float z = 0.f, ss = 0.f;
            for (int i = 0; i < NWV; ++i) {
                z += zred[(slot * (2 * P + 2) + 2 * t + side) * NWV + i];
                ss += zred[(slot * (2 * P + 2) + 2 * P + side) * NWV + i];
            }
            if (unit) z *= unit_scale(ss);
            const float u = tanhf(z);
            const float e = mass_ratio(beta, u);
            const float big = 1.0f / (1.0f + e), small = e / (1.0f + e);
            pq[(slot * 2 * P + c) * 2] = (u >= 0.f) ? big : small;          // mass on the +1 side
            pq[(slot * 2 * P + c) * 2 + 1] = (u >= 0.f) ? small : big;
        }
        __syncthreads();
        if (on) {
            for (int r = c; r < 2 * R; r += TL) {
                const int side = r / R, cr = r % R;
                float f = 1.f;
                for (int t = 0; t < P; ++t) f *= pq[(slot * 2 * P + side * P + t) * 2 + (((cr >> t) & 1) ? 0 : 1)];
                phi[(slot * 2 + side) * R + cr] = f;
            }
        }
        __syncthreads();
        if (on) {
            const float *pqv = phi + (slot * 2) * R, *pk = pqv + R;
            float *S = state + (static_cast<size_t>(bh) * L + l) * R * d1;
            if (c < d) {
#pragma unroll 8
                for (int r = 0; r < R; ++r) {
                    const float sv = fmaf(pk[r], vv, S[r * d1 + c]);
                    S[r * d1 + c] = sv;
                    num = fmaf(pqv[r], sv, num);
                }
            }
            for (int r = c; r < R; r += TL) {       // the mass column
                const float sv = S[r * d1 + d] + pk[r];
                S[r * d1 + d] = sv;
                dn = fmaf(pqv[r], sv, dn);
            }
        }
        __syncthreads();
    }
    if (colok) numred[slot * d + c] = num;
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) dn += __shfl_xor(dn, m, 64);
    if (lane == 0) dred[tid >> 6] = dn;
    __syncthreads();
    if (tid < d) {
        float tot = 0.f, dnt = 0.f;
        for (int sl = 0; sl < TF; ++sl) tot += numred[sl * d + tid];
        for (int i = 0; i < kDecodeThreads / 64; ++i) dnt += dred[i];
        store_elem(o, static_cast<size_t>(bh) * d + tid, dnt > 0.f ? tot / dnt : 0.f);
        if (tid == 0) den[bh] = dnt / static_cast<float>(L);
    }
}

__global__ void zero_kernel(float *dst, size_t n)
{
    const size_t stride = static_cast<size_t>(gridDim.x) * blockDim.x;
    for (size_t i = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = 0.f;
}

// ------------------------------------------------------------------ host side
int pick_tile(int R, int d, int P)
{
    for (int tt = 8; tt >= 1; tt >>= 1)
        if (smem_floats(R, d, P, tt) * sizeof(float) <= 160 * 1024) return tt;
    return 0;
}

Args make_args(const Plan &p, const char *ws)
{
    Args a;
    a.H = p.H; a.L = p.L; a.P = p.P; a.R = p.R; a.d = p.d; a.LP = p.LP;
    a.nseg = p.nseg; a.causal = p.causal; a.TT = pick_tile(p.R, p.d, p.P);
    a.N = p.N; a.seg_len = p.seg_len; a.beta = p.beta; a.unit = p.unit_qk;
    a.W = reinterpret_cast<const float *>(ws + p.off_W);
    return a;
}

template <typename K>
hipError_t allow_lds(K kernel, size_t bytes)
{
    return hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(bytes));
}

#define RACE_TRY(expr)                                   \
    do {                                                 \
        hipError_t e_ = (expr);                          \
        if (e_ != hipSuccess) return e_;                 \
    } while (0)

unsigned blocks_for(size_t n, unsigned per) { return static_cast<unsigned>((n + per - 1) / per); }

template <typename T>
hipError_t fwd_impl(const Plan &p, const T *Q, const T *K, const T *V, T *O, float *den, char *ws, hipStream_t st)
{
    const Args a = make_args(p, ws);
    const size_t lds = smem_floats(p.R, p.d, p.P, a.TT) * sizeof(float);
    float *state = reinterpret_cast<float *>(ws + p.off_stateA);
    float *part = reinterpret_cast<float *>(ws + p.off_part);
    const dim3 grid(p.nseg, p.L, p.BH);
    const size_t elems = static_cast<size_t>(p.R) * (p.d + 1);
    RACE_TRY(allow_lds(simple_totals<T, 0>, lds));
    RACE_TRY(allow_lds(simple_fwd_replay<T>, lds));
    {
        ProfileScope prof("simple_totals_kv", st);
        hipLaunchKernelGGL((simple_totals<T, 0>), grid, dim3(kThreads), lds, st, a, K, V,
                           static_cast<const T *>(nullptr), static_cast<const float *>(nullptr), state);
    }
    {
        ProfileScope prof("simple_scan", st);
        hipLaunchKernelGGL(simple_scan, dim3(blocks_for(elems, 256), p.BH * p.L), dim3(256), 0, st, state, p.nseg,
                           elems, p.causal ? 0 : 2);
    }
    {
        ProfileScope prof("simple_fwd_replay", st);
        hipLaunchKernelGGL((simple_fwd_replay<T>), grid, dim3(kThreads), lds, st, a, Q, K, V, state, part);
    }
    const size_t total = static_cast<size_t>(p.BH) * p.N * p.d;
    {
        ProfileScope prof("simple_fwd_combine", st);
        hipLaunchKernelGGL((simple_fwd_combine<T>), dim3(blocks_for(total, 256)), dim3(256), 0, st, a, p.BH, part, O, den);
    }
    return hipGetLastError();
}

template <typename T>
hipError_t bwd_impl(const Plan &p, const T *Q, const T *K, const T *V, const T *O, const float *den, const T *dO,
                    T *dQ, T *dK, T *dV, float *dbeta, char *ws, hipStream_t st)
{
    const Args a = make_args(p, ws);
    const size_t lds = smem_floats(p.R, p.d, p.P, a.TT) * sizeof(float);
    float *dbeta_part = reinterpret_cast<float *>(ws + p.off_dbeta);
    float *stateS = reinterpret_cast<float *>(ws + p.off_stateA);
    float *stateD = reinterpret_cast<float *>(ws + p.off_stateB);
    float *pQ = reinterpret_cast<float *>(ws + p.off_part);
    const size_t per = static_cast<size_t>(p.BH) * p.L * p.N * p.d;
    float *pK = pQ + per, *pV = pK + per;
    const dim3 grid(p.nseg, p.L, p.BH);
    const size_t elems = static_cast<size_t>(p.R) * (p.d + 1);
    const dim3 sgrid(blocks_for(elems, 256), p.BH * p.L);
    RACE_TRY(allow_lds(simple_totals<T, 0>, lds));
    RACE_TRY(allow_lds(simple_totals<T, 1>, lds));
    RACE_TRY(allow_lds(simple_bwd_query<T>, lds));
    RACE_TRY(allow_lds(simple_bwd_keyvalue<T>, lds));
    {
        ProfileScope prof("simple_totals_kv", st);
        hipLaunchKernelGGL((simple_totals<T, 0>), grid, dim3(kThreads), lds, st, a, K, V,
                           static_cast<const T *>(nullptr), static_cast<const float *>(nullptr), stateS);
    }
    {
        ProfileScope prof("simple_scan", st);
        hipLaunchKernelGGL(simple_scan, sgrid, dim3(256), 0, st, stateS, p.nseg, elems, p.causal ? 0 : 2);
    }
    {
        ProfileScope prof("simple_totals_qg", st);
        hipLaunchKernelGGL((simple_totals<T, 1>), grid, dim3(kThreads), lds, st, a, Q, dO, O, den, stateD);
    }
    {
        ProfileScope prof("simple_scan", st);
        hipLaunchKernelGGL(simple_scan, sgrid, dim3(256), 0, st, stateD, p.nseg, elems, p.causal ? 1 : 2);
    }
    {
        ProfileScope prof("simple_bwd_query", st);
        hipLaunchKernelGGL((simple_bwd_query<T>), grid, dim3(kThreads), lds, st, a, Q, K, V, O, den, dO, stateS, pQ,
                           dbeta_part);
    }
    {
        ProfileScope prof("simple_bwd_keyvalue", st);
        hipLaunchKernelGGL((simple_bwd_keyvalue<T>), grid, dim3(kThreads), lds, st, a, Q, K, V, O, den, dO, stateD, pK,
                           pV, dbeta_part);
    }
    const size_t total = static_cast<size_t>(p.BH) * p.N * p.d;
    {
        ProfileScope prof("simple_bwd_combine", st);
        hipLaunchKernelGGL((simple_bwd_combine<T>), dim3(blocks_for(total, 256)), dim3(256), 0, st, a, p.BH, pQ, pK, pV,
                           dQ, dK, dV);
    }
    if (dbeta) RACE_TRY(reduce_dbeta(p, dbeta_part, dbeta, st));
    return hipGetLastError();
}

// One thread per (batch, head): both sides' partial sums in index order.
__global__ void dbeta_reduce_kernel(const float *part, int BH, int parts, float *dbeta)
{
    const int bh = blockIdx.x * blockDim.x + threadIdx.x;
    if (bh >= BH) return;
    float s = 0.f;
    for (int side = 0; side < 2; ++side) {
        const float *src = part + (static_cast<size_t>(side) * BH + bh) * parts;
        for (int i = 0; i < parts; ++i) s += src[i];
    }
    dbeta[bh] = s;
}

}  // namespace

hipError_t reduce_dbeta(const Plan &p, const float *part, float *dbeta, hipStream_t st)
{
    hipLaunchKernelGGL(dbeta_reduce_kernel, dim3(blocks_for(static_cast<size_t>(p.BH), 64)), dim3(64), 0, st, part,
                       p.BH, p.dbeta_parts, dbeta);
    return hipGetLastError();
}

bool simple_supported(int R, int d, int P) { return pick_tile(R, d, P) > 0; }

hipError_t simple_fwd(const Plan &p, const void *Q, const void *K, const void *V, void *O, float *den, char *ws,
                      hipStream_t st)
{
    if (p.dtype == RACE_F32)
        return fwd_impl<float>(p, (const float *)Q, (const float *)K, (const float *)V, (float *)O, den, ws, st);
    return fwd_impl<bf16_t>(p, (const bf16_t *)Q, (const bf16_t *)K, (const bf16_t *)V, (bf16_t *)O, den, ws, st);
}

hipError_t simple_bwd(const Plan &p, const void *Q, const void *K, const void *V, const void *O, const float *den,
                      const void *dO, void *dQ, void *dK, void *dV, float *dbeta, char *ws, hipStream_t st)
{
    if (p.dtype == RACE_F32)
        return bwd_impl<float>(p, (const float *)Q, (const float *)K, (const float *)V, (const float *)O, den,
                               (const float *)dO, (float *)dQ, (float *)dK, (float *)dV, dbeta, ws, st);
    return bwd_impl<bf16_t>(p, (const bf16_t *)Q, (const bf16_t *)K, (const bf16_t *)V, (const bf16_t *)O, den,
                            (const bf16_t *)dO, (bf16_t *)dQ, (bf16_t *)dK, (bf16_t *)dV, dbeta, ws, st);
}

hipError_t simple_hash(const Plan &p, const void *X, uint8_t *codes, float *phi, char *ws, hipStream_t st)
{
    const Args a = make_args(p, ws);
    const size_t total = static_cast<size_t>(p.BH) * p.N * p.L;
    if (p.dtype == RACE_F32)
        hipLaunchKernelGGL((simple_hash_tap<float>), dim3(blocks_for(total, 128)), dim3(128), 0, st, a, p.BH,
                           (const float *)X, codes, phi);
    else
        hipLaunchKernelGGL((simple_hash_tap<bf16_t>), dim3(blocks_for(total, 128)), dim3(128), 0, st, a, p.BH,
                           (const bf16_t *)X, codes, phi);
    return hipGetLastError();
}

hipError_t zero_floats(float *dst, size_t n, hipStream_t st)
{
    const size_t want = (n + 255) / 256;
    hipLaunchKernelGGL(zero_kernel, dim3(static_cast<unsigned>(want < 4096 ? (want ? want : 1) : 4096)), dim3(256), 0, st,
                       dst, n);
    return hipGetLastError();
}

hipError_t decode_step(const Plan &p, const float *W, const void *q, const void *k, const void *v, float *state,
                       void *o, float *den, hipStream_t st)
{
    const int TL = (p.d + 63) & ~63, TF = kDecodeThreads / TL;
    const size_t lds = (static_cast<size_t>(TF) * (2 * p.P + 2) * (TL / 64) + TF * 4 * p.P + TF * 2 * p.R + TF * p.d + 16) * sizeof(float);
    if (p.dtype == RACE_F32)
        hipLaunchKernelGGL((decode_step_kernel<float>), dim3(p.BH), dim3(kDecodeThreads), lds, st, p.H, p.L, p.P, p.d, p.beta, p.unit_qk, W,
                           (const float *)q, (const float *)k, (const float *)v, state, (float *)o, den);
    else
        hipLaunchKernelGGL((decode_step_kernel<bf16_t>), dim3(p.BH), dim3(kDecodeThreads), lds, st, p.H, p.L, p.P, p.d, p.beta, p.unit_qk, W,
                           (const bf16_t *)q, (const bf16_t *)k, (const bf16_t *)v, state, (bf16_t *)o, den);
    return hipGetLastError();
}

hipError_t simple_buckets(const Plan &p, const void *K, const void *V, float *A, float *Bsum, int a_stride,
                          int b_stride, char *ws, hipStream_t st)
{
    const Args a = make_args(p, ws);
    const size_t lds = smem_floats(p.R, p.d, p.P, a.TT) * sizeof(float);
    float *state = reinterpret_cast<float *>(ws + p.off_stateA);
    const dim3 grid(p.nseg, p.L, p.BH);
    if (p.dtype == RACE_F32) {
        RACE_TRY(allow_lds(simple_totals<float, 0>, lds));
        hipLaunchKernelGGL((simple_totals<float, 0>), grid, dim3(kThreads), lds, st, a, (const float *)K,
                           (const float *)V, (const float *)nullptr, (const float *)nullptr, state);
    } else {
        RACE_TRY(allow_lds(simple_totals<bf16_t, 0>, lds));
        hipLaunchKernelGGL((simple_totals<bf16_t, 0>), grid, dim3(kThreads), lds, st, a, (const bf16_t *)K,
                           (const bf16_t *)V, (const bf16_t *)nullptr, (const float *)nullptr, state);
    }
    const size_t total = static_cast<size_t>(p.BH) * p.L * p.R * (p.d + 1);
    hipLaunchKernelGGL(simple_bucket_tap, dim3(blocks_for(total, 256)), dim3(256), 0, st, a, p.BH, state, A, Bsum,
                       a_stride, b_stride);
    return hipGetLastError();
}

// One 16-byte load and one 16-byte store per element, grid-stride: every byte is read once and written once.
__global__ void __launch_bounds__(256) calibration_copy_kernel(uint4 *__restrict__ dst, const uint4 *__restrict__ src,
                                                                size_t n16)
{
    const size_t stride = static_cast<size_t>(gridDim.x) * blockDim.x;
    for (size_t i = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

hipError_t calibration_copy(void *dst, const void *src, size_t bytes, hipStream_t st)
{
    const size_t n16 = bytes / 16;
    const size_t want = (n16 + 255) / 256;
    const unsigned blocks = static_cast<unsigned>(want < 16384 ? (want ? want : 1) : 16384);
    hipLaunchKernelGGL(calibration_copy_kernel, dim3(blocks), dim3(256), 0, st, static_cast<uint4 *>(dst),
                       static_cast<const uint4 *>(src), n16);
    return hipGetLastError();
}

}  // namespace race
