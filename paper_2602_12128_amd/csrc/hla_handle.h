// The library-owned handle behind the opaque hla_handle of include/hla.h (internal).
#ifndef HLA_HANDLE_H_
#define HLA_HANDLE_H_

#include <vector>

#include "hla_common.h"

// One table of token runs per role (what a kernel family cuts the tokens into); rebuilt in place
// when (B, N, cu_seqlens) or the role's block size changes.  Allocated once, at the capacity the
// role's smallest block size needs.
struct hla_token_table {
  int32_t min_block = 0;            // smallest block size the role ever asks for; 0 = role unused
  int32_t block_tokens = 0;         // block size of the current contents
  hla::BlockEnt* dev = nullptr;     // capacity entries
  int32_t* seq_off_dev = nullptr;   // [max_seqs+1] first block of each sequence
  int64_t capacity = 0;
  int32_t count = 0;                // valid entries for the current shape
  bool valid = false;
};
constexpr int kTableRoles = 3;
constexpr int kVmodWgradParts = 1024;  // most partial sums (workgroups per map) of the modulation's weight gradients

struct hla_call_args {
  int32_t B, H, N;
  int32_t num_seqs;                // effective number of sequences (B when dense)
  bool packed;
  hla::View Q, K, V, O, dO, dQ, dK, dV;
  hipStream_t stream;
};

struct hla_handle {
  hla_config cfg;
  int32_t path;                    // HLA_PATH_GENERIC or HLA_PATH_MFMA
  hla::Geom g;                     // d, dphi, F, D, nfeat, eps filled at create; B,H,N per call
  int64_t max_th;                  // max_heads * max_tokens
  int32_t max_units;               // max_seqs * max_heads

  // device workspace
  float* feat = nullptr;           // [max_th][nfeat]   features saved by forward
  float* dfeat = nullptr;          // [max_th][nfeat]   feature gradients
  float* den = nullptr;            // [max_th]          eta + eps saved by forward
  float* yhat = nullptr;           // path-specific per-token scratch, yhat_floats long
  int64_t yhat_floats = 0;
  float* state = nullptr;          // [max_units][state_stride]
  float* dstate = nullptr;         // [max_units][state_stride]
  float* partial = nullptr;        // [max_chunks * max_heads][state_stride]
  int64_t state_stride = 0;        // floats per (sequence, head) state
  int64_t max_chunks = 0;
  void* path_ws = nullptr;         // extra path-owned device memory (repacked weights, bf16 state)
  size_t path_ws_bytes = 0;
  size_t w_packed_off = 0;         // byte offset of the MFMA path's packed feature-map weights in path_ws
  size_t causal_off = 0;           // byte offset of the per-chunk prefix-state images (causal handles)
  bool causal_partials_valid = false;  // the partial buffer still holds the last causal forward's chunk states
  bool causal_rows_valid = false;      // the monomial-row image of the running state belongs to the last forward
  bool causal_seen_backward = false;   // a backward has run on this handle: forwards prepare that image too
  size_t causal_bwd_off = 0;       // byte offset of the per-chunk state / gradient-state images of the causal backward

  // feature-map weights, fp32 copies (both paths keep them; the MFMA path adds packed bf16)
  float* w_f32 = nullptr;
  hla::PhiF32 phi{};
  bool have_weights = false;

  // weight-gradient outputs (optional): caller's fp32 arrays and the per-workgroup partial sums
  bool wg_on = false;
  hla_phi_weight_grads wg_out[5] = {};
  float* wg_partial = nullptr;     // [wg_parts_cap][wg_part_floats]
  int64_t wg_parts_cap = 0;
  int64_t wg_part_floats = 0;      // d*d + d + d*dphi + dphi

  // value modulation (optional): fp32 weights of the two maps, the saved attention output T, the
  // gradient w.r.t. T and the modulation's share of dV ([max_th][d] in the I/O dtype each)
  bool vmod_on = false;
  float vmod_ln_eps = 0.0f;
  float* vmod_w = nullptr;
  unsigned char* vmod_wpk = nullptr;  // matrix-core kernels' packed copy of the two maps and their scratch (if used)
  void* vmod_T = nullptr;
  void* vmod_dT = nullptr;
  void* vmod_dV = nullptr;
  bool fw_vmod = false;            // mode of the last forward
  // gradients of the modulation's own weights (optional): caller's fp32 arrays, per-workgroup partials
  bool vmod_wg_on = false;
  hla_vmod_weight_grads vmod_wg_out[2] = {};
  float* vmod_wg_partial = nullptr;  // [kVmodWgradParts][d d + d]
  float* vmod_wg_rows = nullptr;     // three [max_th][d] arrays of per-token factors

  // token tables, one per role (the path's workspace plan names the roles it uses)
  hla_token_table tables[kTableRoles];
  // true: the device workspace is carved out of memory the handle does not own (nothing to free)
  bool borrowed_ws = false;
  std::vector<int32_t> cu_host;    // shape signature of the tables (effective cu, B rows if dense)
  int32_t sig_B = -1, sig_N = -1;
  bool sig_packed = false;

  // signature of the last forward, checked by backward
  bool have_forward = false;
  int32_t fw_B = 0, fw_H = 0, fw_N = 0;
  bool fw_packed = false;
  std::vector<int32_t> fw_cu;
  const void *fw_Q = nullptr, *fw_K = nullptr, *fw_V = nullptr;

  hla::Profiler prof;
};

namespace hla {

// Ensure the table of `role` holds runs of `block_tokens` tokens for the current call shape;
// rebuilt on `s` if stale (dense batches: by a kernel; packed sequences: uploaded).
hla_status get_table(hla_handle* hd, int role, int32_t block_tokens, hipStream_t s, hla_token_table** out);

template <typename... KArgs, typename... Args>
inline hla_status launch(hla_handle* hd, const char* name, void (*kernel)(KArgs...), dim3 grid,
                         dim3 block, size_t shmem, hipStream_t s, Args... args) {
  if (grid.x == 0 || grid.y == 0 || grid.z == 0) return HLA_OK;
  hd->prof.begin(name, s);
  kernel<<<grid, block, shmem, s>>>(static_cast<KArgs>(args)...);
  hd->prof.end(s);
  return hipGetLastError() == hipSuccess ? HLA_OK : HLA_ERR_HIP;
}

// Path entry points (hla_generic.hip / hla_mfma.hip).
hla_status generic_workspace_plan(hla_handle* hd);
hla_status generic_set_weights(hla_handle* hd, hipStream_t s);
hla_status generic_forward(hla_handle* hd, const hla_call_args& a);
hla_status generic_backward(hla_handle* hd, const hla_call_args& a);
hla_status generic_features_in(hla_handle* hd, const hla_call_args& a);
hla_status generic_features_out(hla_handle* hd, const hla_call_args& a);

bool mfma_supported(const hla_config& c);
hla_status mfma_workspace_plan(hla_handle* hd);
// Launch attributes (LDS sizes above the default limit) of the kernels this handle will launch,
// on the current device.
hla_status mfma_prepare_kernels(const hla_handle* hd);
hla_status generic_prepare_kernels(const hla_handle* hd);
hla_status mfma_phi_prepare_kernels(const hla_handle* hd);
hla_status mfma_set_weights(hla_handle* hd, hipStream_t s);
hla_status mfma_forward(hla_handle* hd, const hla_call_args& a);
hla_status mfma_backward(hla_handle* hd, const hla_call_args& a);

// Feature maps on matrix cores (hla_mfma_phi.hip).
size_t mfma_phi_packed_bytes(const hla_handle* hd);
hla_status mfma_phi_set_weights(hla_handle* hd, hipStream_t s);
hla_status mfma_phi_forward(hla_handle* hd, const hla_call_args& a);
hla_status mfma_phi_backward(hla_handle* hd, const hla_call_args& a);

// Value modulation (hla_vmod.hip): weights into hd->vmod_w; O = T + phi_v1(T) * phi_v2(V) from
// hd->vmod_T and a.V into a.O; (a.dO, T, V) -> hd->vmod_dT, hd->vmod_dV; a.dV += hd->vmod_dV.
hla_status vmod_set_weights(hla_handle* hd, const hla_vmod_weights* maps, hipStream_t s);
hla_status vmod_forward(hla_handle* hd, const hla_call_args& a);
hla_status vmod_backward(hla_handle* hd, const hla_call_args& a);
hla_status vmod_add_value_grads(hla_handle* hd, const hla_call_args& a);
View vmod_view(void* p, const Geom& g);  // contiguous [B, H, N, d] view of a workspace array
// Gradients of the modulation's weights from (hd->vmod_T, a.V, a.dO = gradient w.r.t. the modulated
// output) into the registered arrays; `empty`: no tokens, zeros are written.
hla_status vmod_weight_grads(hla_handle* hd, const hla_call_args& a, bool empty);
int64_t vmod_wgrad_part_floats(int d);
// The same on the matrix cores (hla_mfma_vmod.hip), used by the functions above where supported.
bool vmod_mfma_supported(const hla_handle* hd);
size_t vmod_mfma_packed_bytes(const hla_handle* hd);
size_t vmod_mfma_workspace_bytes(const hla_handle* hd);  // packed weights + what the forward keeps per tile for the backward
hla_status vmod_mfma_prepare_kernels(const hla_handle* hd);
hla_status vmod_mfma_set_weights(hla_handle* hd, const hla_vmod_weights* maps, hipStream_t s);
hla_status vmod_mfma_forward(hla_handle* hd, const hla_call_args& a);
hla_status vmod_mfma_backward(hla_handle* hd, const hla_call_args& a);
hla_status vmod_mfma_add_value_grads(hla_handle* hd, const hla_call_args& a);
hla_status vmod_mfma_weight_grads(hla_handle* hd, const hla_call_args& a);
int64_t vmod_mfma_factor_floats(const hla_handle* hd);
int64_t vmod_mfma_partial_floats(const hla_handle* hd);

// Shared helper kernels' host wrappers (hla_generic.hip).
hla_status convert_weights_to_f32(hla_handle* hd, const hla_phi_weights* maps, hipStream_t s);
// Weight gradients of the feature maps from the saved features and feature gradients: partial
// sums by the path's kernel (matrix cores where the MFMA path has one, else the fp32 kernel of
// hla_generic.hip), then weight_grads_reduce adds `nparts` partials per (map, head) in order,
// scales the four sections and writes the caller's arrays.
hla_status phi_weight_grads(hla_handle* hd, const hla_call_args& a);
hla_status mfma_phi_weight_grads(hla_handle* hd, const hla_call_args& a);
hla_status weight_grads_reduce(hla_handle* hd, int nparts, int heads, float sW1, float sb1, float sW2,
                               float sb2, hipStream_t s);

}  // namespace hla

#define HLA_TRY(expr)                   \
  do {                                  \
    hla_status _s = (expr);             \
    if (_s != HLA_OK) return _s;        \
  } while (0)

#endif  // HLA_HANDLE_H_
