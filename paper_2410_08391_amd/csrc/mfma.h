// bf16 MFMA kernels (gfx950 matrix cores) for the auxiliary prefill and the predictor.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <vector>
#include "../../include/kvp.h"
#include "common.h"

namespace kvp {

// accessors into the opaque handle (defined in kvp_api.hip)
const std::vector<const void*>& handle_pred_wk(const kvp_handle* h);
const std::vector<const void*>& handle_pred_wv(const kvp_handle* h);
const std::vector<int32_t>& handle_layer_map(const kvp_handle* h);
const kvp_config& handle_cfg(const kvp_handle* h);

// per-handle device tables of the predictor kernels (built by mfma_prepare)
struct MfmaTables {
  const bf16** w_tab = nullptr;   // device [2 * L_B]: W_K,i at 2i, W_V,i at 2i+1
  int32_t* layer_map = nullptr;   // device [L_B]
};

// true if every shape of the configuration fits the MFMA kernels' tiling
bool mfma_supported(const kvp_config* cfg);                 // the auxiliary stack of cfg
bool mfma_shape_supported(const kvp_model_shape* m);        // any decoder stack
size_t mfma_vt_bytes_shape(const kvp_model_shape* m, int B, int T_len);
// per-handle device tables (predictor weight pointers, layer map); released by mfma_release
int mfma_prepare(kvp_handle* h, void** tables_out);
void mfma_release(void* tables);
// bytes of the transposed value buffer the attention kernel reads
size_t mfma_vt_bytes(const kvp_config* cfg, int B, int T_len);

// q/k/v = h W^T for head_dim 128 heads, rotary on q and k;  q -> [N, n_q*128],  k, v -> [N, n_kv*128],
// and v also transposed into vT [B][n_kv][128][round_up(T, 64)] when vT != NULL.  wq may be NULL
// (then q is not computed).  With rotate == false q and k are stored unrotated (a query / key
// normalisation follows and rotates afterwards).
void mfma_qkv_rope(const bf16* hbuf, const bf16* wq, const bf16* wk, const bf16* wv, bf16* q, bf16* k, bf16* v, bf16* vT,
                   int N, int d, int n_q, int n_kv, int T_len, const float2* rope_tab, bool rotate, hipStream_t s);
// causal grouped-query flash attention (head_dim 128): q, k token-major, v from the transposed copy
void mfma_flash_prefill(const bf16* q, const bf16* k, const bf16* vT, bf16* out, int B, int T_len, int n_q, int n_kv,
                        hipStream_t s);
// overflow guard of the attention kernels' fixed-reference softmax, for the whole process (0: the default)
void mfma_set_flash_guard(float limit);
// X[M,N] += A[M,K] W[N,K]^T  (float32 residual stream)
void mfma_gemm_residual(const bf16* A, const bf16* W, float* X, int M, int N, int K, hipStream_t s);
// act[M,F] = silu(A Wg^T) * (A Wu^T)
void mfma_gemm_swiglu(const bf16* A, const bf16* Wg, const bf16* Wu, bf16* act, int M, int F, int K, hipStream_t s);
// predicted K/V of base layers [layer0, layer1) in one launch, written in the base cache layout.
// The layers share one auxiliary layer (Ka wide) and one width Kb = n_kv_b * head_dim; aux_block /
// layer_elems are the element strides between the auxiliary layers' and the cache layers' blocks.
int mfma_predictor(const kvp_handle* h, void* tables, const bf16* aux_k, const bf16* aux_v, bf16* k_cache,
                   bf16* v_cache, int B, int T_len, int64_t T_cap, int layer0, int layer1, int Ka, int Kb, int n_kv_b,
                   size_t aux_block, size_t layer_elems, hipStream_t s);

// The same result from the streaming kernel (kernels_predictor.hip: tokens stationary in registers,
// weights streamed through LDS, base layers of [layer0, layer1) grouped into runs that share an
// auxiliary layer).  Returns false, with nothing launched, for shapes it does not serve
// (Ka other than 256 / 512, base head_dim other than 128, short prompts).
bool mfma_predictor_stream(const kvp_handle* h, void* tables, const bf16* aux_k, const bf16* aux_v, bf16* k_cache,
                           bf16* v_cache, int B, int T_len, int64_t T_cap, int layer0, int layer1, int Ka, int Kb,
                           int n_kv_b, size_t aux_block, size_t layer_elems, hipStream_t s);

}  // namespace kvp
