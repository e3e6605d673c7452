// Internal declarations shared by the translation units of the library (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "race_attn.h"

namespace race {

constexpr int kFamilyNone = 0;
constexpr int kFamilySimple = 1;   // generic kernels, fp32 arithmetic on the vector ALUs
constexpr int kFamilyMfma = 2;     // bf16 MFMA kernels, register-resident bucket state

// Everything the launchers need, derived once from a validated descriptor.
struct Plan {
    int B, H, BH, d, L, P, R, LP, LR;
    // MFMA family: the compiled shape that serves the problem (Lc >= L tables, Pc >= P hyperplanes; the padding
    // tables are empty and the padding hyperplanes put all mass on one side); equal to L, P, LR otherwise
    int Lc, Pc, LRc;
    int pad;            // 1: the padded instantiation of the compiled shape serves the problem
    int64_t N;
    float beta;
    int causal;
    int unit_qk;        // rows of Q and K are divided by their norms before the projection
    int dtype;
    int family;
    // The sequence is cut into nseg segments of seg_len tokens (the last may be short).  One
    // workgroup owns one segment; segment totals of the bucket statistics are turned into
    // segment-start states by an exclusive scan (forward: prefix, backward: suffix).
    int nseg;
    int64_t seg_len;
    // workspace layout, byte offsets (all multiples of 256)
    size_t off_W;       // projection matrix in the layout of the kernel family
    size_t bytes_W;
    size_t off_stateA;  // per-segment bucket statistics, (BH, nseg, ...) fp32
    size_t off_stateB;  // second set (backward only: cotangent statistics)
    size_t bytes_state;
    size_t off_part;    // per-table partial results (simple family only)
    size_t bytes_part;
    size_t off_massQ;   // MFMA family: the hashed rows of Q and of K, (BH, N, Lc * Pc) fp32 each (one float per token,
    size_t off_massK;   // table and hyperplane: the per-bit soft-hash masses every pass rebuilds phi from)
    size_t bytes_mass;
    size_t fwd_bytes;   // the leading part of the workspace that the forward pass uses
    size_t off_dbeta;   // partial cotangents of beta: (2 sides, BH, dbeta_parts) fp32, backward only
    size_t bytes_dbeta;
    int dbeta_parts;    // partial sums per (side, batch*head): one per workgroup of the gradient kernels
    size_t total;
    // backward only: the workspace still holds the forward's projection image, hashed rows and segment-start
    // key/value statistics (set by race_attn_bwd_saved for the families that can use them)
    int fwd_state_kept;
};

// Validates desc and fills plan.  Returns RACE_OK, RACE_ERR_INVALID_ARG or RACE_ERR_UNSUPPORTED.
race_status_t make_plan(const race_attn_desc_t *desc, Plan *plan);

// Host: pinned, immutable image of W for (seeds, L, P, d, dtype) in the layout of `family`.  Images live until the
// process ends (a pending asynchronous copy or a captured graph may still read one), so the pointer stays valid.
// may_allocate == false: only looks the image up.  Returns nullptr if the image is not there and may not be made,
// if the cache is full (kMaxProjectionImages distinct keys) or if pinned memory cannot be allocated; *why then
// names the reason (static string).
constexpr size_t kMaxProjectionImages = 4096;
const void *projection_image(const Plan &plan, const uint64_t *seeds, size_t *bytes, bool may_allocate, const char **why);

// The library's own device scratch for race_attn_fwd_static (static_scratch.hip): a fixed array in the code object.
constexpr size_t kStaticScratchBytes = static_cast<size_t>(32) << 20;
hipError_t static_scratch(void **ptr);     // device address of the current device's copy
// Host: plain (H, L*P, d) expansion into caller memory.
void expand_projection_host(int H, int L, int P, int d, int dtype, const uint64_t *seeds, float *out);

// Brackets one kernel launch with HIP events on its stream while profiling is enabled (benchmark aid).
struct ProfileScope {
    ProfileScope(const char *name, hipStream_t st);
    ~ProfileScope();
    void *rec_;
    hipStream_t st_;
};

// dbeta[bh] = sum over the two sides and the dbeta_parts partial sums of part, in index order (simple_kernels.hip).
hipError_t reduce_dbeta(const Plan &p, const float *part, float *dbeta, hipStream_t st);

// Plain copy of known size (simple_kernels.hip); bytes is a multiple of 16.
hipError_t calibration_copy(void *dst, const void *src, size_t bytes, hipStream_t st);
// Dense bf16 MFMA loop on register operands (mfma_kernels.hip).
hipError_t calibration_mfma(int workgroups, int iters, int vector_ops, float *sink, hipStream_t st);

// ---- simple family (simple_kernels.hip)
hipError_t simple_fwd(const Plan &p, const void *Q, const void *K, const void *V, void *O, float *den,
                      char *ws, hipStream_t st);
hipError_t simple_bwd(const Plan &p, const void *Q, const void *K, const void *V, const void *O,
                      const float *den, const void *dO, void *dQ, void *dK, void *dV, float *dbeta, char *ws,
                      hipStream_t st);
hipError_t simple_hash(const Plan &p, const void *X, uint8_t *codes, float *phi, char *ws, hipStream_t st);
// A[(bh*L*R + row) * a_stride] and Bsum[(bh*L*R + row) * b_stride + column]: separate tensors (1, d) or one
// interleaved (B, H, L, R, d+1) state (A = state + d, Bsum = state, both strides d+1)
hipError_t simple_buckets(const Plan &p, const void *K, const void *V, float *A, float *Bsum, int a_stride,
                          int b_stride, char *ws, hipStream_t st);
// One decoding step (simple_kernels.hip): W fp32 (H, L*P, d) and partial (BH, L, d+1) in the workspace.
hipError_t decode_step(const Plan &p, const float *W, const void *q, const void *k, const void *v, float *state,
                       void *o, float *den, hipStream_t st);
hipError_t zero_floats(float *dst, size_t n, hipStream_t st);

// ---- MFMA family (mfma_kernels.hip, mfma_grad.hip).  Compiled shapes: X(d, P, L)
// X(d, P, L, PAD): PAD = 0 serves exactly that shape, PAD = 1 also everything smaller in L and P
#ifndef RACE_MFMA_SHAPES
#define RACE_MFMA_SHAPES(X) X(128, 6, 8, 0) X(64, 4, 16, 0) X(64, 4, 16, 1) X(128, 4, 16, 1) X(128, 6, 8, 1) X(64, 6, 8, 1) X(128, 4, 4, 1) X(128, 4, 8, 1)
#endif
// The exact shape if compiled, else the padded instantiation with the fewest bucket rows that covers (d, L, P).
bool mfma_pick(int d, int L, int P, int *Lc, int *Pc, int *pad);
size_t mfma_hashed_bytes(const Plan &p);       // bytes of the hashed rows of one tensor
size_t mfma_projection_bytes(const Plan &p);
void mfma_pack_projection(const Plan &p, const float *W, void *image);   // host
hipError_t mfma_fwd(const Plan &p, const void *Q, const void *K, const void *V, void *O, float *den,
                    char *ws, hipStream_t st);
hipError_t mfma_bwd(const Plan &p, const void *Q, const void *K, const void *V, const void *O,
                    const float *den, const void *dO, void *dQ, void *dK, void *dV, float *dbeta, char *ws,
                    hipStream_t st);
int mfma_dbeta_parts(const Plan &p);           // workgroups per (side, batch*head) of the gradient kernels
hipError_t mfma_hash(const Plan &p, const void *X, uint8_t *codes, float *phi, char *ws, hipStream_t st);
hipError_t mfma_buckets(const Plan &p, const void *K, const void *V, float *A, float *Bsum, int a_stride,
                        int b_stride, char *ws, hipStream_t st);

}  // namespace race
