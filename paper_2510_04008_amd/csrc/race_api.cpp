// Host side of the C ABI: argument validation, planning (segments, workspace layout), the
// seed -> W generator with its host cache, and dispatch to the kernel families.
#include <hip/hip_runtime_api.h>

#include <cmath>
#include <cstdlib>
#include <cstring>
#include <map>
#include <mutex>
#include <string>
#include <vector>

#include "internal.h"

namespace race {

bool simple_supported(int R, int d, int P);

namespace {

thread_local std::string g_last_error;

// largest per-table partial-result area the generic kernels are offered (their workspace grows like L * N * d)
constexpr size_t kGenericPartialLimit = static_cast<size_t>(16) << 30;

size_t align256(size_t x) { return (x + 255) & ~static_cast<size_t>(255); }

// ---------------------------------------------------------------- Philox-4x32-10 + Box-Muller
// Counter-based generator of Salmon et al. (SC'11): ten rounds of two 32x32->64 multiplications,
// the key bumped by the Weyl constants between rounds.
struct Philox4 { uint32_t v[4]; };

Philox4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0, uint32_t k1)
{
    for (int round = 0; round < 10; ++round) {
        if (round) { k0 += 0x9E3779B9u; k1 += 0xBB67AE85u; }
        const uint64_t a = 0xD2511F53ull * c0, b = 0xCD9E8D57ull * c2;
        const uint32_t n0 = static_cast<uint32_t>(b >> 32) ^ c1 ^ k0;
        const uint32_t n2 = static_cast<uint32_t>(a >> 32) ^ c3 ^ k1;
        c1 = static_cast<uint32_t>(b);
        c3 = static_cast<uint32_t>(a);
        c0 = n0;
        c2 = n2;
    }
    return Philox4{{c0, c1, c2, c3}};
}

void gaussian_pair(uint32_t x0, uint32_t x1, double *g)
{
    const double u1 = (static_cast<double>(x0) + 0.5) * (1.0 / 4294967296.0);
    const double u2 = (static_cast<double>(x1) + 0.5) * (1.0 / 4294967296.0);
    const double rad = std::sqrt(-2.0 * std::log(u1));
    const double ang = 2.0 * 3.14159265358979323846 * u2;
    g[0] = rad * std::cos(ang);
    g[1] = rad * std::sin(ang);
}

float round_to_bf16(float x)
{
    uint32_t b;
    std::memcpy(&b, &x, 4);
    b += 0x7fffu + ((b >> 16) & 1u);
    b &= 0xffff0000u;
    std::memcpy(&x, &b, 4);
    return x;
}

// ---------------------------------------------------------------- host cache of projection images
struct CacheKey {
    int family, dtype, H, L, P, d;
    std::vector<uint64_t> seeds;
    bool operator<(const CacheKey &o) const
    {
        if (family != o.family) return family < o.family;
        if (dtype != o.dtype) return dtype < o.dtype;
        if (H != o.H) return H < o.H;
        if (L != o.L) return L < o.L;
        if (P != o.P) return P < o.P;
        if (d != o.d) return d < o.d;
        return seeds < o.seeds;
    }
};
struct CacheEntry { void *pinned; size_t bytes; };
std::mutex g_cache_mutex;
std::map<CacheKey, CacheEntry> g_cache;

}  // namespace

void expand_projection_host(int H, int L, int P, int d, int dtype, const uint64_t *seeds, float *out)
{
    const size_t n = static_cast<size_t>(L) * P * d;
    for (int h = 0; h < H; ++h) {
        const uint32_t k0 = static_cast<uint32_t>(seeds[h]), k1 = static_cast<uint32_t>(seeds[h] >> 32);
        float *w = out + static_cast<size_t>(h) * n;
        for (size_t blk = 0; blk * 4 < n; ++blk) {
            const Philox4 x = philox4x32_10(static_cast<uint32_t>(blk), static_cast<uint32_t>(blk >> 32), 0, 0, k0, k1);
            double g[4];
            gaussian_pair(x.v[0], x.v[1], g);
            gaussian_pair(x.v[2], x.v[3], g + 2);
            for (size_t i = 0; i < 4 && blk * 4 + i < n; ++i) {
                float f = static_cast<float>(g[i]);
                w[blk * 4 + i] = (dtype == RACE_BF16) ? round_to_bf16(f) : f;
            }
        }
    }
}

// An image is never freed or moved once made: an asynchronous copy that was enqueued from it, or a captured graph
// that holds such a copy, may read it at any later time.  The cache is therefore bounded by refusing new keys, not
// by evicting old ones (an image is a few KB to ~100 KB).
const void *projection_image(const Plan &p, const uint64_t *seeds, size_t *bytes, bool may_allocate, const char **why)
{
    CacheKey key{p.family, p.dtype, p.H, p.L, p.P, p.d, std::vector<uint64_t>(seeds, seeds + p.H)};
    std::lock_guard<std::mutex> lock(g_cache_mutex);
    auto it = g_cache.find(key);
    if (it == g_cache.end()) {
        if (!may_allocate) {
            *why = "the projection image of these seeds and this shape has not been prepared by an earlier call";
            return nullptr;
        }
        if (g_cache.size() >= kMaxProjectionImages) {
            *why = "projection image cache full (4096 distinct combinations of seeds and shape in this process)";
            return nullptr;
        }
        std::vector<float> W(static_cast<size_t>(p.H) * p.LP * p.d);
        expand_projection_host(p.H, p.L, p.P, p.d, p.dtype, seeds, W.data());
        CacheEntry e;
        e.bytes = p.bytes_W;
        if (hipHostMalloc(&e.pinned, e.bytes, hipHostMallocDefault) != hipSuccess) {
            *why = "hipHostMalloc(projection image) failed";
            return nullptr;
        }
        if (p.family == kFamilyMfma) mfma_pack_projection(p, W.data(), e.pinned);
        else std::memcpy(e.pinned, W.data(), W.size() * sizeof(float));
        it = g_cache.emplace(std::move(key), e).first;
    }
    *bytes = it->second.bytes;
    return it->second.pinned;
}

// ---------------------------------------------------------------- per-kernel timing (benchmark aid)
namespace {
struct ProfileRecord { const char *name; hipEvent_t start, stop; };
thread_local bool g_profile_on = false;
thread_local std::vector<ProfileRecord> g_profile_records;
thread_local std::vector<hipEvent_t> g_profile_pool;

hipEvent_t take_event()
{
    if (!g_profile_pool.empty()) {
        hipEvent_t e = g_profile_pool.back();
        g_profile_pool.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    (void)hipEventCreate(&e);
    return e;
}
}  // namespace

ProfileScope::ProfileScope(const char *name, hipStream_t st) : rec_(nullptr), st_(st)
{
    if (!g_profile_on) return;
    ProfileRecord r{name, take_event(), take_event()};
    if (!r.start || !r.stop) return;
    (void)hipEventRecord(r.start, st);
    g_profile_records.push_back(r);
    rec_ = reinterpret_cast<void *>(g_profile_records.size());      // index + 1
}

ProfileScope::~ProfileScope()
{
    if (!rec_) return;
    const size_t i = reinterpret_cast<size_t>(rec_) - 1;
    if (i < g_profile_records.size()) (void)hipEventRecord(g_profile_records[i].stop, st_);
}

race_status_t make_plan(const race_attn_desc_t *desc, Plan *pl)
{
    if (!desc) return RACE_ERR_INVALID_ARG;
    if (desc->B < 1 || desc->H < 1 || desc->N < 0 || desc->d < 1 || desc->L < 1 || desc->P < 1)
        return RACE_ERR_INVALID_ARG;
    if (!(desc->sharpening > 0.0f)) return RACE_ERR_INVALID_ARG;         // NaN fails too; +infinity = hard hash
    if (desc->causal != 0 && desc->causal != 1) return RACE_ERR_INVALID_ARG;
    if (desc->dtype != RACE_F32 && desc->dtype != RACE_BF16) return RACE_ERR_INVALID_ARG;
    if (desc->chunk < 0) return RACE_ERR_INVALID_ARG;
    if (desc->unit_qk != 0 && desc->unit_qk != 1) return RACE_ERR_INVALID_ARG;
    if (desc->P > 8 || desc->d > 256 || desc->d % 8 != 0) return RACE_ERR_UNSUPPORTED;
    if (desc->L > 4096 || static_cast<int64_t>(desc->B) * desc->H > 65535) return RACE_ERR_UNSUPPORTED;
    if (static_cast<int64_t>(desc->B) * desc->H * desc->L > 65535) return RACE_ERR_UNSUPPORTED;
    if (desc->N > (static_cast<int64_t>(1) << 40)) return RACE_ERR_UNSUPPORTED;

    Plan p{};
    p.B = desc->B; p.H = desc->H; p.BH = desc->B * desc->H; p.d = desc->d; p.L = desc->L; p.P = desc->P;
    p.R = 1 << desc->P; p.LP = p.L * p.P; p.LR = p.L * p.R; p.N = desc->N; p.beta = desc->sharpening;
    p.causal = desc->causal; p.dtype = desc->dtype; p.unit_qk = desc->unit_qk;

    const char *force = std::getenv("RACE_ATTN_FORCE_GENERIC");
    const bool forced = force && force[0] == '1';
    p.Lc = p.L; p.Pc = p.P; p.LRc = p.LR; p.pad = 0;
    if (p.dtype == RACE_BF16 && !forced && mfma_pick(p.d, p.L, p.P, &p.Lc, &p.Pc, &p.pad)) {
        p.family = kFamilyMfma;
        p.LRc = p.Lc * (1 << p.Pc);
    } else if (simple_supported(p.R, p.d, p.P)) p.family = kFamilySimple;
    else return RACE_ERR_UNSUPPORTED;

    const int64_t n = p.N > 0 ? p.N : 1;
    if (p.family == kFamilySimple) {
        // enough workgroups to fill 256 CUs a few times over, segments of at least 16 tokens (the kernels take the
        // tokens of a segment one after the other: short sequences want many short segments)
        int64_t want = (2048 + static_cast<int64_t>(p.BH) * p.L - 1) / (static_cast<int64_t>(p.BH) * p.L);
        int64_t len = desc->chunk > 0 ? desc->chunk : (n + want - 1) / want;
        if (desc->chunk == 0 && len < 16) len = 16;
        len = (len + 7) / 8 * 8;
        p.seg_len = len;
        p.nseg = static_cast<int>((n + len - 1) / len);
        if ((n + len - 1) / len > 65535) return RACE_ERR_UNSUPPORTED;
        p.bytes_W = align256(static_cast<size_t>(p.H) * p.LP * p.d * sizeof(float));
        p.bytes_state = align256(static_cast<size_t>(p.BH) * p.L * p.nseg * p.R * (p.d + 1) * sizeof(float));
        const size_t fwd_part = static_cast<size_t>(p.BH) * p.L * n * (p.d + 1) * sizeof(float);
        const size_t bwd_part = static_cast<size_t>(p.BH) * p.L * n * p.d * sizeof(float) * 3;
        p.bytes_part = align256(fwd_part > bwd_part ? fwd_part : bwd_part);
        // these kernels keep per-table partial results of every token in the workspace (L * N * d floats): they are
        // the fp32 reference path, not a long-context path
        if (p.bytes_part > kGenericPartialLimit) return RACE_ERR_UNSUPPORTED;
        p.dbeta_parts = p.L * p.nseg;
    } else {
        // two workgroups' worth of segments per CU and head-batch; multiples of the 32-token tile
        int64_t want = (512 + p.BH - 1) / p.BH;
        int64_t len = desc->chunk > 0 ? desc->chunk : (n + want - 1) / want;
        if (desc->chunk == 0 && len < 256) len = 256;
        len = (len + 31) / 32 * 32;
        p.seg_len = len;
        if ((n + len - 1) / len > 65535) return RACE_ERR_UNSUPPORTED;
        p.nseg = static_cast<int>((n + len - 1) / len);
        p.bytes_W = align256(mfma_projection_bytes(p));
        p.bytes_state = align256(static_cast<size_t>(p.BH) * p.nseg * p.LRc * (p.d + 1) * sizeof(float));
        p.bytes_part = 0;
        p.bytes_mass = align256(mfma_hashed_bytes(p));
        p.dbeta_parts = mfma_dbeta_parts(p);
    }
    p.bytes_dbeta = align256(static_cast<size_t>(2) * p.BH * p.dbeta_parts * sizeof(float));
    // [W | key/value statistics | hashed Q | hashed K] is what the forward pass uses (and leaves behind);
    // [cotangent statistics | per-table partial results | parts of dbeta] follow
    p.off_W = 0;
    p.off_stateA = p.off_W + p.bytes_W;
    p.off_massQ = p.off_stateA + p.bytes_state;
    p.off_massK = p.off_massQ + p.bytes_mass;
    p.off_stateB = p.off_massK + p.bytes_mass;
    p.off_part = p.off_stateB + p.bytes_state;
    p.off_dbeta = p.off_part + p.bytes_part;
    p.total = p.off_dbeta + p.bytes_dbeta;
    p.fwd_bytes = (p.family == kFamilyMfma) ? p.off_stateB : p.off_dbeta;
    *pl = p;
    return RACE_OK;
}

namespace {

race_status_t hip_failed(hipError_t e, const char *where)
{
    g_last_error = std::string(where) + ": " + hipGetErrorString(e);
    return RACE_ERR_HIP;
}

race_status_t check_workspace(const Plan &p, const void *ws, size_t bytes, size_t need)
{
    (void)p;
    if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255) != 0 || bytes < need) return RACE_ERR_WORKSPACE;
    return RACE_OK;
}

bool any_equal(std::initializer_list<const void *> outs, std::initializer_list<const void *> all)
{
    for (const void *o : outs) {
        int hits = 0;
        for (const void *a : all) hits += (a == o);
        if (hits > 1) return true;
    }
    return false;
}

race_status_t upload_projection(const Plan &p, const uint64_t *seeds, char *ws, hipStream_t st, bool may_allocate = true)
{
    size_t bytes = 0;
    const char *why = "";
    const void *img = projection_image(p, seeds, &bytes, may_allocate, &why);
    if (!img) {
        g_last_error = why;
        return may_allocate ? RACE_ERR_HIP : RACE_ERR_NOT_READY;
    }
    hipError_t e = hipMemcpyAsync(ws + p.off_W, img, bytes, hipMemcpyHostToDevice, st);
    if (e != hipSuccess) return hip_failed(e, "hipMemcpyAsync(projection image)");
    return RACE_OK;
}

}  // namespace
}  // namespace race

using namespace race;

extern "C" {

size_t race_attn_workspace_bytes(const race_attn_desc_t *desc)
{
    Plan p;
    if (make_plan(desc, &p) != RACE_OK || p.N == 0) return 0;
    return p.total;
}

int race_attn_kernel_family(const race_attn_desc_t *desc)
{
    Plan p;
    if (make_plan(desc, &p) != RACE_OK) return kFamilyNone;
    return p.family;
}

int64_t race_attn_segment_tokens(const race_attn_desc_t *desc)
{
    Plan p;
    if (make_plan(desc, &p) != RACE_OK) return 0;
    return p.seg_len;
}

race_status_t race_attn_fwd(const race_attn_desc_t *desc, const void *Q, const void *K, const void *V,
                            const uint64_t *proj_seeds, void *O, float *den, void *workspace,
                            size_t workspace_bytes, race_stream_t stream)
{
    Plan p;
    race_status_t s = make_plan(desc, &p);
    if (s != RACE_OK) return s;
    if (p.N == 0) return RACE_OK;      // nothing to do, pointers may be null
    if (!Q || !K || !V || !proj_seeds || !O || !den) return RACE_ERR_INVALID_ARG;
    if (any_equal({O, den}, {Q, K, V, O, den})) return RACE_ERR_INVALID_ARG;
    if ((s = check_workspace(p, workspace, workspace_bytes, p.total)) != RACE_OK) return s;
    char *ws = static_cast<char *>(workspace);
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if ((s = upload_projection(p, proj_seeds, ws, st)) != RACE_OK) return s;
    hipError_t e = (p.family == kFamilyMfma) ? mfma_fwd(p, Q, K, V, O, den, ws, st)
                                             : simple_fwd(p, Q, K, V, O, den, ws, st);
    return e == hipSuccess ? RACE_OK : hip_failed(e, "race_attn_fwd launch");
}

// The forward pass on the library's own scratch array: same kernels, same arguments, no allocation of any kind.
race_status_t race_attn_fwd_static(const race_attn_desc_t *desc, const void *Q, const void *K, const void *V,
                                   const uint64_t *proj_seeds, void *O, float *den, race_stream_t stream)
{
    Plan p;
    race_status_t s = make_plan(desc, &p);
    if (s != RACE_OK) return s;
    if (p.N == 0) return RACE_OK;
    if (!Q || !K || !V || !proj_seeds || !O || !den) return RACE_ERR_INVALID_ARG;
    if (any_equal({O, den}, {Q, K, V, O, den})) return RACE_ERR_INVALID_ARG;
    // Fewer, longer scan segments until the forward's share of the workspace (W, the segment statistics and, for the
    // generic kernels, the per-table partial results) fits the array; a caller's own desc->chunk is kept as the
    // smallest segment length tried.
    race_attn_desc_t fit = *desc;
    for (;;) {
        if (p.fwd_bytes <= kStaticScratchBytes) break;
        if (p.nseg <= 1) {
            g_last_error = "race_attn_fwd_static: the problem needs more than the 32 MiB of built-in scratch; use race_attn_fwd with a workspace";
            return RACE_ERR_WORKSPACE;
        }
        fit.chunk = p.seg_len * 2;
        if ((s = make_plan(&fit, &p)) != RACE_OK) return s;
    }
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    // the image must be there already: making it would allocate pinned host memory
    size_t bytes = 0;
    const char *why = "";
    if (!projection_image(p, proj_seeds, &bytes, false, &why)) {
        g_last_error = std::string("race_attn_fwd_static: ") + why;
        return RACE_ERR_NOT_READY;
    }
    void *scratch = nullptr;
    hipError_t e = static_scratch(&scratch);
    if (e != hipSuccess) return hip_failed(e, "hipGetSymbolAddress(static scratch)");
    char *ws = static_cast<char *>(scratch);
    if ((s = upload_projection(p, proj_seeds, ws, st, false)) != RACE_OK) return s;
    e = (p.family == kFamilyMfma) ? mfma_fwd(p, Q, K, V, O, den, ws, st) : simple_fwd(p, Q, K, V, O, den, ws, st);
    return e == hipSuccess ? RACE_OK : hip_failed(e, "race_attn_fwd_static launch");
}

race_status_t race_attn_bwd(const race_attn_desc_t *desc, const void *Q, const void *K, const void *V,
                            const void *O, const float *den, const void *dO, const uint64_t *proj_seeds,
                            void *dQ, void *dK, void *dV, void *workspace, size_t workspace_bytes,
                            race_stream_t stream)
{
    return race_attn_bwd_beta(desc, Q, K, V, O, den, dO, proj_seeds, dQ, dK, dV, nullptr, workspace, workspace_bytes,
                              stream);
}

namespace {
race_status_t backward(const race_attn_desc_t *desc, const void *Q, const void *K, const void *V, const void *O,
                       const float *den, const void *dO, const uint64_t *proj_seeds, void *dQ, void *dK, void *dV,
                       float *dbeta, void *workspace, size_t workspace_bytes, race_stream_t stream, bool saved);
}

race_status_t race_attn_bwd_beta(const race_attn_desc_t *desc, const void *Q, const void *K, const void *V,
                                 const void *O, const float *den, const void *dO, const uint64_t *proj_seeds,
                                 void *dQ, void *dK, void *dV, float *dbeta, void *workspace,
                                 size_t workspace_bytes, race_stream_t stream)
{
    return backward(desc, Q, K, V, O, den, dO, proj_seeds, dQ, dK, dV, dbeta, workspace, workspace_bytes, stream, false);
}

race_status_t race_attn_bwd_saved(const race_attn_desc_t *desc, const void *Q, const void *K, const void *V,
                                  const void *O, const float *den, const void *dO, const uint64_t *proj_seeds,
                                  void *dQ, void *dK, void *dV, float *dbeta, void *workspace,
                                  size_t workspace_bytes, race_stream_t stream)
{
    return backward(desc, Q, K, V, O, den, dO, proj_seeds, dQ, dK, dV, dbeta, workspace, workspace_bytes, stream, true);
}

namespace {
race_status_t backward(const race_attn_desc_t *desc, const void *Q, const void *K, const void *V, const void *O,
                       const float *den, const void *dO, const uint64_t *proj_seeds, void *dQ, void *dK, void *dV,
                       float *dbeta, void *workspace, size_t workspace_bytes, race_stream_t stream, bool saved)
{
    Plan p;
    race_status_t s = make_plan(desc, &p);
    if (s != RACE_OK) return s;
    if (p.N == 0) return RACE_OK;      // nothing to do, pointers may be null
    if (!Q || !K || !V || !O || !den || !dO || !proj_seeds || !dQ || !dK || !dV) return RACE_ERR_INVALID_ARG;
    if (std::isinf(p.beta)) return RACE_ERR_UNSUPPORTED;      // the hard hash is piecewise constant: inference only
    if (any_equal({dQ, dK, dV}, {Q, K, V, O, den, dO, dQ, dK, dV})) return RACE_ERR_INVALID_ARG;
    if (dbeta && any_equal({dbeta}, {Q, K, V, O, den, dO, dQ, dK, dV, dbeta})) return RACE_ERR_INVALID_ARG;
    if ((s = check_workspace(p, workspace, workspace_bytes, p.total)) != RACE_OK) return s;
    char *ws = static_cast<char *>(workspace);
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    // the MFMA family's forward leaves its projection image and segment-start statistics where the backward
    // pass looks for them; the generic family's forward reuses that area for other things and starts over
    p.fwd_state_kept = (saved && p.family == kFamilyMfma) ? 1 : 0;
    if (!p.fwd_state_kept && (s = upload_projection(p, proj_seeds, ws, st)) != RACE_OK) return s;
    hipError_t e = (p.family == kFamilyMfma) ? mfma_bwd(p, Q, K, V, O, den, dO, dQ, dK, dV, dbeta, ws, st)
                                             : simple_bwd(p, Q, K, V, O, den, dO, dQ, dK, dV, dbeta, ws, st);
    return e == hipSuccess ? RACE_OK : hip_failed(e, "race_attn_bwd launch");
}
}  // namespace

race_status_t race_attn_expand_projection(const race_attn_desc_t *desc, const uint64_t *proj_seeds, float *W_host)
{
    if (!desc || !proj_seeds || !W_host) return RACE_ERR_INVALID_ARG;
    if (desc->H < 1 || desc->L < 1 || desc->P < 1 || desc->d < 1) return RACE_ERR_INVALID_ARG;
    if (desc->dtype != RACE_F32 && desc->dtype != RACE_BF16) return RACE_ERR_INVALID_ARG;
    if (desc->P > 8 || desc->d > 256 || desc->L > 4096) return RACE_ERR_UNSUPPORTED;
    expand_projection_host(desc->H, desc->L, desc->P, desc->d, desc->dtype, proj_seeds, W_host);
    return RACE_OK;
}

race_status_t race_attn_debug_hash(const race_attn_desc_t *desc, const void *X, const uint64_t *proj_seeds,
                                   uint8_t *codes, float *phi, void *workspace, size_t workspace_bytes,
                                   race_stream_t stream)
{
    Plan p;
    race_status_t s = make_plan(desc, &p);
    if (s != RACE_OK) return s;
    if (p.N == 0) return RACE_OK;      // nothing to do, pointers may be null
    if (!X || !proj_seeds || !codes) return RACE_ERR_INVALID_ARG;
    if ((s = check_workspace(p, workspace, workspace_bytes, p.off_W + p.bytes_W)) != RACE_OK) return s;
    char *ws = static_cast<char *>(workspace);
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if ((s = upload_projection(p, proj_seeds, ws, st)) != RACE_OK) return s;
    hipError_t e = (p.family == kFamilyMfma) ? mfma_hash(p, X, codes, phi, ws, st)
                                             : simple_hash(p, X, codes, phi, ws, st);
    return e == hipSuccess ? RACE_OK : hip_failed(e, "race_attn_debug_hash launch");
}

race_status_t race_attn_debug_buckets(const race_attn_desc_t *desc, const void *K, const void *V,
                                      const uint64_t *proj_seeds, float *A, float *Bsum, void *workspace,
                                      size_t workspace_bytes, race_stream_t stream)
{
    Plan p;
    race_status_t s = make_plan(desc, &p);
    if (s != RACE_OK) return s;
    if (p.N == 0) return RACE_OK;      // nothing to do, pointers may be null
    if (!K || !V || !proj_seeds || !A || !Bsum) return RACE_ERR_INVALID_ARG;
    if ((s = check_workspace(p, workspace, workspace_bytes, p.total)) != RACE_OK) return s;
    char *ws = static_cast<char *>(workspace);
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if ((s = upload_projection(p, proj_seeds, ws, st)) != RACE_OK) return s;
    hipError_t e = (p.family == kFamilyMfma) ? mfma_buckets(p, K, V, A, Bsum, 1, p.d, ws, st)
                                             : simple_buckets(p, K, V, A, Bsum, 1, p.d, ws, st);
    return e == hipSuccess ? RACE_OK : hip_failed(e, "race_attn_debug_buckets launch");
}

size_t race_attn_state_bytes(const race_attn_desc_t *desc)
{
    Plan p;
    race_attn_desc_t one;
    if (!desc) return 0;
    one = *desc;
    one.N = 1;                             // the state does not depend on the context length
    if (one.chunk < 0) one.chunk = 0;
    if (make_plan(&one, &p) != RACE_OK) return 0;
    return static_cast<size_t>(p.BH) * p.LR * (p.d + 1) * sizeof(float);
}

race_status_t race_attn_state_init(const race_attn_desc_t *desc, const void *K, const void *V,
                                   const uint64_t *proj_seeds, float *state, void *workspace,
                                   size_t workspace_bytes, race_stream_t stream)
{
    Plan p;
    race_status_t s = make_plan(desc, &p);
    if (s != RACE_OK) return s;
    if (!state) return RACE_ERR_INVALID_ARG;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if (p.N == 0) {                        // empty context
        hipError_t e = zero_floats(state, static_cast<size_t>(p.BH) * p.LR * (p.d + 1), st);
        return e == hipSuccess ? RACE_OK : hip_failed(e, "race_attn_state_init launch");
    }
    if (!K || !V || !proj_seeds) return RACE_ERR_INVALID_ARG;
    if (static_cast<const void *>(state) == K || static_cast<const void *>(state) == V) return RACE_ERR_INVALID_ARG;
    if ((s = check_workspace(p, workspace, workspace_bytes, p.total)) != RACE_OK) return s;
    char *ws = static_cast<char *>(workspace);
    if ((s = upload_projection(p, proj_seeds, ws, st)) != RACE_OK) return s;
    // interleaved layout: per bucket row d sums, then the mass
    hipError_t e = (p.family == kFamilyMfma) ? mfma_buckets(p, K, V, state + p.d, state, p.d + 1, p.d + 1, ws, st)
                                             : simple_buckets(p, K, V, state + p.d, state, p.d + 1, p.d + 1, ws, st);
    return e == hipSuccess ? RACE_OK : hip_failed(e, "race_attn_state_init launch");
}

namespace {
// A decoding step runs on the generic kernels' fp32 image of W whatever family serves the long passes.
race_status_t make_step_plan(const race_attn_desc_t *desc, Plan *pl)
{
    if (!desc) return RACE_ERR_INVALID_ARG;
    race_attn_desc_t one = *desc;
    one.N = 1;
    one.causal = 1;
    one.chunk = 0;
    race_status_t s = make_plan(&one, pl);
    if (s != RACE_OK) return s;
    pl->family = kFamilySimple;
    pl->off_W = 0;
    pl->bytes_W = align256(static_cast<size_t>(pl->H) * pl->LP * pl->d * sizeof(float));
    pl->off_part = pl->bytes_W;
    pl->bytes_part = 0;
    pl->total = pl->off_part + pl->bytes_part;
    return RACE_OK;
}
}  // namespace

size_t race_attn_step_workspace_bytes(const race_attn_desc_t *desc)
{
    Plan p;
    return make_step_plan(desc, &p) == RACE_OK ? p.total : 0;
}

race_status_t race_attn_step(const race_attn_desc_t *desc, const void *q, const void *k, const void *v,
                             const uint64_t *proj_seeds, float *state, void *o, float *den, void *workspace,
                             size_t workspace_bytes, race_stream_t stream)
{
    Plan p;
    race_status_t s = make_step_plan(desc, &p);
    if (s != RACE_OK) return s;
    if (!q || !k || !v || !state || !o || !den) return RACE_ERR_INVALID_ARG;
    if (any_equal({state, o, den}, {q, k, v, state, o, den})) return RACE_ERR_INVALID_ARG;
    if ((s = check_workspace(p, workspace, workspace_bytes, p.total)) != RACE_OK) return s;
    char *ws = static_cast<char *>(workspace);
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    // no seeds: the workspace still holds the W that an earlier step put there
    if (proj_seeds && (s = upload_projection(p, proj_seeds, ws, st)) != RACE_OK) return s;
    hipError_t e = decode_step(p, reinterpret_cast<const float *>(ws + p.off_W), q, k, v, state, o, den, st);
    return e == hipSuccess ? RACE_OK : hip_failed(e, "race_attn_step launch");
}

const char *race_status_string(race_status_t status)
{
    switch (status) {
    case RACE_OK: return "ok";
    case RACE_ERR_INVALID_ARG: return "invalid argument";
    case RACE_ERR_UNSUPPORTED: return "unsupported shape";
    case RACE_ERR_WORKSPACE: return "workspace null, misaligned or too small";
    case RACE_ERR_HIP: return "HIP call failed";
    case RACE_ERR_NOT_READY: return "a call that prepares this one has not been made";
    }
    return "unknown status";
}

const char *race_attn_last_error(void) { return g_last_error.c_str(); }

race_status_t race_attn_calibration_copy(void *dst, const void *src, size_t bytes, race_stream_t stream)
{
    if (bytes == 0) return RACE_OK;
    if (!dst || !src || bytes % 16 != 0) return RACE_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(dst) % 16 != 0 || reinterpret_cast<uintptr_t>(src) % 16 != 0)
        return RACE_ERR_INVALID_ARG;
    const char *a = static_cast<const char *>(src);
    const char *b = static_cast<const char *>(dst);
    if (a < b + bytes && b < a + bytes) return RACE_ERR_INVALID_ARG;
    hipError_t e = calibration_copy(dst, src, bytes, reinterpret_cast<hipStream_t>(stream));
    if (e != hipSuccess) {
        g_last_error = std::string("calibration_copy: ") + hipGetErrorString(e);
        return RACE_ERR_HIP;
    }
    return RACE_OK;
}

race_status_t race_attn_calibration_mfma(int workgroups, int iters, int vector_ops, float *sink, race_stream_t stream)
{
    if (!sink || workgroups < 1 || iters < 1 || workgroups > (1 << 20) || iters > (1 << 20)) return RACE_ERR_INVALID_ARG;
    if (vector_ops != 0 && vector_ops != 4 && vector_ops != 8 && vector_ops != 16) return RACE_ERR_INVALID_ARG;
    hipError_t e = calibration_mfma(workgroups, iters, vector_ops, sink, reinterpret_cast<hipStream_t>(stream));
    if (e != hipSuccess) {
        g_last_error = std::string("calibration_mfma: ") + hipGetErrorString(e);
        return RACE_ERR_HIP;
    }
    return RACE_OK;
}

void race_attn_profile_enable(int on)
{
    g_profile_on = on != 0;
    if (!on) {
        for (auto &r : g_profile_records) { g_profile_pool.push_back(r.start); g_profile_pool.push_back(r.stop); }
        g_profile_records.clear();
    }
}

int race_attn_profile_read(int max_entries, const char **names, float *total_ms, int *launches)
{
    std::vector<const char *> seen;
    std::vector<float> ms;
    std::vector<int> cnt;
    for (auto &r : g_profile_records) {
        float t = 0.f;
        if (hipEventSynchronize(r.stop) == hipSuccess) (void)hipEventElapsedTime(&t, r.start, r.stop);
        size_t k = 0;
        while (k < seen.size() && std::strcmp(seen[k], r.name) != 0) ++k;
        if (k == seen.size()) { seen.push_back(r.name); ms.push_back(0.f); cnt.push_back(0); }
        ms[k] += t;
        cnt[k] += 1;
        g_profile_pool.push_back(r.start);
        g_profile_pool.push_back(r.stop);
    }
    g_profile_records.clear();
    for (size_t k = 0; k < seen.size() && static_cast<int>(k) < max_entries; ++k) {
        if (names) names[k] = seen[k];
        if (total_ms) total_ms[k] = ms[k];
        if (launches) launches[k] = cnt[k];
    }
    return static_cast<int>(seen.size());
}

}  // extern "C"
