// Internal declarations shared by the host orchestration and the kernel files.
// Nothing here is part of the ABI (see include/tgrad.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/tgrad.h"

namespace tgrad {

constexpr int kMaxNdim = TGRAD_MAX_NDIM;

// ---- selection (Algorithm 1: SparseIndices) -------------------------------------------------
// A "segment" is the run of consecutive elements one wavefront turns into mask bits; a "chunk" is
// the run one wavefront counts and emits in order from the masks.
constexpr int kSegElems = 2048;
constexpr int kSelChunkElems = 32768;
constexpr int kHistBins = 4096;            // 12-bit digits; the three digits are 12 + 12 + 8 bits

struct SelectScalars {                     // lives in workspace, written by the pick kernel
  uint32_t prefix;                         // key bits fixed so far (high-aligned digits)
  uint32_t remaining;                      // how many entries are still to take inside `prefix`
  uint32_t threshold;                      // final: key of the k-th largest entry
  uint32_t need_eq;                        // final: entries with key == threshold to take (lowest indices)
};

// ---- one mode-n product stage: Out[a, m, b] = sum_k F[m, k] X[a, k, b] ------------------------
struct Stage {
  int mode;                                // which tensor mode this stage contracts
  int64_t A;                               // product of the extents left of the mode
  int K;                                   // extent being contracted
  int M;                                   // extent produced
  int64_t B;                               // product of the extents right of the mode
};

// Names of the profiled kernels (index into the per-context timing table).
enum KernelId {
  KID_SEL_HIST = 0, KID_SEL_PICK, KID_SEL_SPLIT, KID_SEL_HIST_CAND, KID_SEL_COUNT, KID_SEL_SCAN, KID_SEL_EMIT,
  KID_MASK_FROM_IDX,
  KID_TILE_OFFSETS, KID_GRAM, KID_GRAM_REDUCE, KID_EIG, KID_FACTOR_PACK,
  KID_GATHER, KID_PROJECT_FIRST, KID_PROJECT, KID_ADAM_CORE, KID_BACKPROJECT, KID_UPDATE,
  KID_SPARSE_UPDATE, KID_HOOI_PROJECT, KID_CORE, KID_RESIDUAL, KID_COUNT
};

struct Launch {                            // what every launcher needs
  hipStream_t stream;
};

// selection.  SelectKeys: random == false -> keys are |g|^2 of the gradient; true -> keys are the
// index hash built from the two words (the gradient pointer is then unused).
struct SelectKeys {
  bool random;
  uint32_t s0, s1;
};
void launch_select_hist(hipStream_t s, const void* g, int dtype, const SelectKeys& keys, int64_t I,
                        uint32_t* hist);
void launch_select_pick(hipStream_t s, int pass, uint32_t k, SelectScalars* sc, const uint32_t* hist);
void launch_select_split(hipStream_t s, const void* g, int dtype, const SelectKeys& keys, int64_t I,
                         const SelectScalars* sc, uint32_t* sure, uint32_t* cand);
void launch_select_hist_cand(hipStream_t s, const void* g, int dtype, const SelectKeys& keys, int64_t I,
                             int pass, const SelectScalars* sc, const uint32_t* cand, uint32_t* hist);
void launch_select_count(hipStream_t s, const void* g, int dtype, const SelectKeys& keys, int64_t I,
                         const SelectScalars* sc, const uint32_t* sure, const uint32_t* cand,
                         uint32_t* chunk_gt, uint32_t* chunk_eq, int64_t nchunks);
void launch_select_scan(hipStream_t s, uint32_t* chunk_gt, uint32_t* chunk_eq, int64_t nchunks);
void launch_select_emit(hipStream_t s, const void* g, int dtype, const SelectKeys& keys, int64_t I,
                        const SelectScalars* sc, const uint32_t* chunk_gt, const uint32_t* chunk_eq,
                        int64_t nchunks, uint32_t* sure, const uint32_t* cand, int32_t* omega);
void launch_mask_from_indices(hipStream_t s, const int32_t* omega, int64_t k, uint32_t* mask,
                              int64_t mask_words);

// factor refresh
int gram_num_chunks(int64_t A, int In, int64_t B);
size_t eig_work_bytes(int n);                      // size of launch_eig_batch's per-mode buffer work_a
void launch_gram(hipStream_t s, const void* g, int dtype, const uint32_t* mask, int64_t A, int In,
                 int64_t B, int nchunks, double* partials);
void launch_gram_reduce(hipStream_t s, const double* partials, int nchunks, int In, double* gram);
void launch_eig(hipStream_t s, const double* gram, double* work_a, double* work_v, int In, int r,
                float* U);

// step
void launch_gather(hipStream_t s, const void* g, int dtype, const int32_t* omega, int64_t k,
                   float2* out);
void launch_contract(hipStream_t s, const void* x, int x_dtype, const uint32_t* mask,
                     const float2* U, int In, int rn, bool project, const Stage& st, float2* out);
void launch_adam_core(hipStream_t s, const float2* r, float2* m, float* v, float2* n_out, int64_t C,
                      float beta1, float beta2, float inv_c1, float inv_c2, float eps);
void launch_sparse_adam(hipStream_t s, float2* gs, int64_t k, float2* m, float* v, float beta1, float beta2,
                        float inv_c1, float inv_c2, float eps, float neg_lr_lambda);
void launch_update(hipStream_t s, const float2* z, const float2* U, int In, int rn, const Stage& st, void* w,
                   int wdtype, float decay, float neg_lr_alpha, const uint32_t* mask, const int32_t* omega,
                   int64_t k, const float2* ns);

void launch_residual(hipStream_t s, const void* g, int dtype, const float2* z, const float2* U, int rn, int64_t A,
                     int M, float2* r);
void launch_residual_gather(hipStream_t s, float2* gs, const int32_t* omega, int64_t k, const float2* z,
                            const float2* U, int rn, int M);

// matrix-core kernels of the step (contract_mfma.hip)
int choose_tile_waves(int Klast, int rlast, int prefer);
double launch_mfma_probe(hipStream_t s, int kind, int64_t iters, float* sink);   // returns the launch's flops
int fused_max_last_extent();                       // largest I_N the fused first-stage kernel takes
void launch_tile_offsets(hipStream_t s, const int32_t* omega, int64_t k, int64_t tile_elems,
                         int64_t ntiles, uint32_t* tile_start);
void launch_mid(hipStream_t s, const float2* x, const float2* U, int rn, bool project, const Stage& st,
                float2* out);
bool core_kernel_fits(int K, int M);
void launch_core(hipStream_t s, const float2* x, const float2* U, int rn, int K, int M, int64_t B, float2* m,
                 float* v, float2* g_out, float beta1, float beta2, float inv_c1, float inv_c2, float eps,
                 float2* z);
int core2_kernel_vec(int I0, int I1, int M0, int M1, int K2, int K);   // columns per workgroup (2, 1) or 0
size_t core2_table_bytes(int I1);
void launch_pack_core2(hipStream_t s, const float2* U0, int rn0, int M0, const float2* U1, int rn1, int M1, int I1,
                       float2* tab);
void launch_core2(hipStream_t s, int vec, int zgroup, const float2* x, const float2* tab, int I1, int M0, int M1, int64_t Cc,
                  float2* m, float* v, float2* g_out, float beta1, float beta2, float inv_c1, float inv_c2,
                  float eps, float2* z);
void launch_pack_fused_factor(hipStream_t s, const float2* U, int I2, int r, float2* fpad, float2* ut);
void launch_lproj(hipStream_t s, const void* g, int dtype, const int32_t* omega, const uint32_t* tile_start,
                  float2* gs, const float2* U, int rn, const Stage& st, int W, float2* out, int fused_I2,
                  int fused_M2, const float2* fpad);
void launch_lupdate(hipStream_t s, const float2* z, const float2* U, const Stage& st, int W, void* w,
                    int wdtype, float decay, float c_alpha, const int32_t* omega, const uint32_t* tile_start,
                    const float2* gs, float2* ms, float* vs, float beta1, float beta2, float inv_c1,
                    float inv_c2, float eps, float c_lambda);

void launch_lupdate_fused(hipStream_t s, const float2* y1, const float2* ut, int I2, int K2, const float2* U,
                          const Stage& st, void* w, int wdtype, float decay, float c_alpha, const int32_t* omega,
                          const uint32_t* tile_start, int64_t k, const float2* gs, float2* ms, float* vs,
                          float beta1, float beta2, float inv_c1, float inv_c2, float eps, float c_lambda,
                          int group);

}  // namespace tgrad
