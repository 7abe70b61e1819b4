// Internal declarations shared by the libmixkv translation units (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "mixkv.h"

namespace mixkv {

constexpr int kWave = 64;
constexpr int kTileKeys = 32;          // keys per MFMA tile
constexpr int kLayersPerLaunch = 32;   // pointer-table entries that fit in one kernel-argument block
constexpr int kSelectThreads = 1024;
constexpr int kMaxCandPerHead = 1024;   // head-adaptive budgets: candidates a head hands to the budget split
constexpr int kMaxCandPerGroup = 4096;  // ... and all heads of one (layer, batch item) together
constexpr int kMaxStreamGrid = 1024;    // upper bound on the workgroups of a streaming kernel launch

// Per-layer device pointers handed to the kernels by value.
struct LayerIn {
  const void *K, *V, *Q;
  int64_t sb, sh, sn;                  // K/V strides in elements
  const float *r_given;                // caller's head weights (mix mode GIVEN_R), else null
};
struct LayerInTable { LayerIn l[kLayersPerLaunch]; };

// The window rows' log-sum-exp per layer, when the caller has it (else all null).
struct LseTable { const float *l[kLayersPerLaunch]; };

struct LayerOut {
  float *scores;                       // may point into the workspace
  float *redundancy;                   // may be null
  int32_t *indices, *counts, *offsets; // offsets may be null (fixed mode)
  void *K_out, *V_out;
};
struct LayerOutTable { LayerOut l[kLayersPerLaunch]; };

// Problem shape, identical for every layer of a call.
struct Shape {
  int32_t batch, hq, hkv, G, D, N, W, Nc, B, Bp;   // Bp = B - W
  int32_t GW;            // G * W query rows per KV head
  int32_t QT;            // ceil(GW / 32) query tiles
  int32_t chunk;         // keys per workgroup in the two streaming kernels
  int32_t nchunks;       // ceil(N / chunk)
  int32_t Npad;          // nchunks * chunk, row length of the per-unit float arrays
  int32_t units_per_layer;
  int32_t nb_rows;       // row length of the per-unit exponent offsets: QT*32 rounded up to 256
  int32_t pool, pool_k, causal, intrinsic, mix, adaptive, per_head, floor_;
  int32_t kstats;        // 1 / |K_i|, the mean normalised key and r are needed (else nothing reads them: the
                         // importance-only mix without the key-norm intrinsic score and without a redundancy output)
  float scale_log2e;     // softmax_scale * log2(e)
  float eps;
};

// Workspace carve-up (byte offsets from a 256-byte aligned base).  Sizes are per call (all units).
struct Workspace {
  size_t budgets;        // int32  [layers][hkv]             per-head budget mode: the caller's table (first, so
                         //                                  that selection alone can run on a workspace this small)
  size_t part_ml;        // float2 [slots][QT*32]            per-run (max, sum) of each softmax row, log2 domain
  size_t part_ksum;      // float  [slots][D]                per-run partial sums of normalised keys
  size_t rbar;           // float  [units]
  size_t nb;             // float  [units][nb_rows]          -b_r per window-query row (-inf past G*W)
  size_t kbarp;          // uint4  [units][64]               mean normalised key as MFMA operand pieces
  size_t invnorm;        // float  [units][Npad]             1 / |K_i|
  size_t vnorm;          // float  [units][Npad]             |V_i|
  size_t araw;           // float  [units][Npad]             window/group mean attention before pooling
  size_t sdiv;           // float  [units][Npad]             K_i . Kbar (the mix kernel applies -1/|K_i|)
  size_t cand_idx;       // int32  [units][kMaxCandPerHead]  adaptive mode: every head's best candidates, ascending
  size_t cand_key;       // uint32 [units][kMaxCandPerHead]  ... and their order-preserving keys
  size_t scores;         // float  [units][N]                used when the caller passes no scores buffer
  size_t total;
};

mixkv_status make_shape(const mixkv_params *p, Shape *s);
void carve_workspace(const Shape &s, int64_t units, Workspace *w, bool select_only = false);

// Kernel launchers (one per pipeline stage).  `unit0` is the first unit of this launch group,
// `nunits` the number of units it covers (whole layers).
// `grid` (from stream_grid) is the number of workgroups of the two streaming kernels; `slot0` is the
// first partial slot of this launch group (each group owns kMaxStreamGrid + its units).
int stream_grid(const Shape &s, int nunits, int num_cus);
// `given_lse`: the caller supplies the softmax normalisers, so the first pass takes key and value
// statistics only; `lse` then holds them per layer (all null otherwise).
hipError_t launch_stats(const Shape &s, int dtype, const LayerInTable &in, char *ws, const Workspace &w, int64_t unit0,
                        int nunits, int grid, int64_t slot0, bool given_lse, hipStream_t st);
// Folds the first pass's per-run partials per unit (exponent offsets, mean key, redundancy).  `grid`
// and `items_per_unit` describe the work split of the first-pass kernel that wrote them.
hipError_t launch_fold(const Shape &s, int dtype, const LayerOutTable &out, const LseTable &lse, char *ws, const Workspace &w,
                       int64_t unit0, int nunits, int grid, int items_per_unit, int64_t slot0, hipStream_t st);
hipError_t launch_attn(const Shape &s, int dtype, const LayerInTable &in, const LayerOutTable &out, const LseTable &lse,
                       char *ws, const Workspace &w, int64_t unit0, int nunits, int grid, int64_t slot0, hipStream_t st);
hipError_t launch_mix(const Shape &s, const LayerInTable &in, const LayerOutTable &out, char *ws, const Workspace &w,
                      int64_t unit0, int nunits, hipStream_t st);
// Weights of s_imp and of the scaled diversity in s_comp (Sec. 3.3, Eq. 5; Table 4's variants);
// r is the head's redundancy, rg the caller's weight.
__device__ __forceinline__ void mix_weights(int mix, float r, float rg, float &wi, float &wd) {
  switch (mix) {
    case MIXKV_MIX_SUM: wi = 1.f; wd = 1.f; break;
    case MIXKV_MIX_DIV_ONLY: wi = 0.f; wd = 1.f; break;
    case MIXKV_MIX_IMP_ONLY: wi = 1.f; wd = 0.f; break;
    case MIXKV_MIX_GIVEN_R: wi = 1.f - rg; wd = rg; break;
    default: wi = 1.f - r; wd = r; break;
  }
}
// |K_i| from its stored reciprocal (0 for a key that normalises to the zero vector).
__device__ __forceinline__ float neg_key_norm(float inv_norm) { return inv_norm > 0.f ? -1.f / inv_norm : 0.f; }
// `budgets` (per-head budget mode, else null): device table [layers of this launch][hkv].
hipError_t launch_select(const Shape &s, const LayerOutTable &out, int nlayers, const int32_t *budgets, hipStream_t st);
// Copies `n` ints from host memory to device memory through kernel arguments (no memcpy, so the
// call neither synchronises nor depends on how the host memory was allocated).
hipError_t upload_ints(const int32_t *host, int n, int32_t *dev, hipStream_t st);
// Head-adaptive budget split from the per-head candidate lists (cand_m entries each) in the workspace.
int adaptive_candidates(const Shape &s);   // cand_m, or 0 if the lists would be too long
hipError_t launch_select_candidates(const Shape &s, const LayerOutTable &out, char *ws, const Workspace &w, int64_t unit0,
                                    int nlayers, int cand_m, hipStream_t st);
hipError_t launch_gather(const Shape &s, int dtype, const LayerInTable &in, const LayerOutTable &out, int nlayers,
                         hipStream_t st);

}  // namespace mixkv
