// Host-side launchers of the gfx950 kernels (one per step of the forward/backward path).
// Each enqueues on `s` and returns hipGetLastError(); none allocates or synchronises.
#pragma once
#include "vsa_common.h"

namespace vsa {

hipError_t launch_tile_permute(const Geo& g, int BH, int H_blhd, int d, const void* src, void* dst, bool inverse,
                               hipStream_t s);
hipError_t launch_mfma_rate(const void* operands, float* sink, int workgroups, int iters, hipStream_t s);
// tensors = 3: Q, K, V pooled per cube; 1: Q only (with launch_pool_keys16 for K and V)
hipError_t launch_pool(const Geo& g, int BH, int d, uint64_t* mask, const void* q, const void* k, const void* v,
                       float* qc, float* kc, float* vc, int tensors, hipStream_t s);
// key cubes of 16 tokens: kc, vc [BH, 4 Nc, d], kcnt [4 Nc] valid tokens per key cube (needs `mask`)
hipError_t launch_pool_keys16(int BH, int Nc, int d, const uint64_t* mask, int32_t* kcnt, const void* k, const void* v,
                              float* kc, float* vc, hipStream_t s);
// Nq query cubes, Nk key cubes; kcnt (or NULL): valid tokens per key cube, 0 = dead
hipError_t launch_coarse(int BH, int Nq, int Nk, int d, int K, float scale, const float* qc, const float* kc,
                         const float* vc, float* sc, float* oc, float* lse_c, int32_t* idx, int emit_idx, int fused,
                         const int32_t* kcnt, hipStream_t s);
hipError_t launch_fine_fwd(int BH, int Nc, int d, int K, float scale, const void* q, const void* k, const void* v,
                           const void* gate_c, const void* gate_f, const int32_t* idx, const float* oc,
                           const uint64_t* mask, void* out, void* out_fine, float* lse_f, int H, int out_token_major,
                           int m_blocks, int key_cubes_16, hipStream_t s);
// lists of cubes -> lists of 64-row blocks, for cubes of m blocks: every block of query cube c gets
// the m blocks of each of the cube's K key cubes, ascending ([BH,Nc,K] -> [BH,Nc*m,K*m])
// mismatched granularity: top-K on the coarse map pooled over (1,2,2) cubes, and its lists of tiles
// turned into lists of cubes for every query cube ([BH,Ns,K] -> [BH,Nc,4K])
hipError_t launch_pooled_select(int BH, int Nt, int Nh, int Nw, int K, const float* P, float* ps, int32_t* tile_idx,
                                hipStream_t s);
hipError_t launch_expand_tiles(int BH, int Nt, int Nh, int Nw, int K, const int32_t* tile_idx, int32_t* idx_blocks,
                               hipStream_t s);
hipError_t launch_expand_lists(int BH, int Nc, int K, int m, const int32_t* idx, int32_t* idx_blocks, hipStream_t s);

// backward
hipError_t launch_bwd_pre(int BH, int Nc, int m_blocks, int d, const uint64_t* mask, const void* dout, const void* gate_c,
                          const void* gate_f, const void* out_fine, const float* oc, void* dgate_c, void* dgate_f,
                          void* dof, float* ld, void* ldb, float scale, float* doc, const float* lse_f, int H,
                          int dout_token_major, hipStream_t s);
hipError_t launch_coarse_bwd(int BH, int Nq, int Nk, int d, float scale, const float* qc, const float* kc,
                             const float* vc, const float* lse_c, const float* doc, float* ac, float* dsc, float* dqc,
                             float* dkc, float* dvc, const int32_t* kcnt, hipStream_t s);
hipError_t launch_transpose_map(int BH, int Nc, int K, const int32_t* idx, uint32_t* bits, int32_t* row_ptr,
                                int32_t* col, int32_t* order, int32_t* split, int seg, int cap, int key_cubes_16,
                                hipStream_t s);
hipError_t launch_fine_bwd_dq(int BH, int Nc, int d, int K, float scale, const void* q, const void* k, const void* v,
                              const void* dof, const int32_t* idx, const float* ld,
                              const float* dqc, const uint64_t* mask, void* dq, int m_blocks, int key_cubes_16,
                              hipStream_t s);
hipError_t launch_fine_bwd_dkv(int BH, int Nc, int d, int K, float scale, const void* q, const void* k, const void* v,
                               const void* dof, const int32_t* col, const int32_t* order, const int32_t* split,
                               float* parts, int cap, const void* ldb, const float* dkc, const float* dvc,
                               const uint64_t* mask, void* dk, void* dv, int m_blocks, int key_cubes_16, hipStream_t s);

}  // namespace vsa
