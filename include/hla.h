/*
 * libhla — non-causal Hadamard Linear Attention (HLA) for AMD MI355X (gfx950).
 *
 * The operator (paper Sec. 4.1, Eq. "hla"; normaliser and factorized evaluation Sec. 4.2,
 * Theorem 4.2; feature maps App. A.1 and Alg. 1 Steps 4-5):
 *
 *     A_ij  = prod_{f=1..F} < phi_q(q_i), phi_kf(k_j) >          (Hadamard product of F score matrices)
 *     eta_i = sum_j A_ij
 *     o_i   = sum_j A_ij v_j / (eta_i + eps)
 *
 * evaluated in O(N) through the key-side state  C = sum_j T_k,j (x) v_j,  z = sum_j T_k,j  with
 * T_k,j = phi_k1(k_j) (x) ... (x) phi_kF(k_j), and the query-side contraction with
 * T_q,i = phi_q(q_i) (x) ... (x) phi_q(q_i).  The N x N matrix is never formed.
 *
 * Plain C ABI: no C++ or torch types cross this boundary.  Unless stated otherwise every
 * tensor pointer is a DEVICE pointer owned by the caller; the library owns only the handle and
 * the workspace inside it.  All work is enqueued on the HIP stream passed in; no entry point
 * synchronises the device except hla_create / hla_destroy.  Failures are returned as codes;
 * nothing is printed and nothing is thrown.  A handle must not be used from two streams or two
 * host threads at the same time.
 */
#ifndef HLA_H_
#define HLA_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct hla_handle hla_handle; /* opaque, library-owned */

typedef enum {
  HLA_OK = 0,
  HLA_ERR_INVALID_ARG = 1, /* null pointer, negative size, bad cu_seqlens, size above the handle's maxima */
  HLA_ERR_UNSUPPORTED = 2, /* (F, d_phi, d, dtype, strides) combination no kernel covers */
  HLA_ERR_ALLOC = 3,       /* hipMalloc / host allocation failed */
  HLA_ERR_HIP = 4,         /* a HIP runtime call failed (launch, copy) */
  HLA_ERR_STATE = 5,       /* call order: backward without weights, weights in PHI_NONE mode, ... */
  HLA_ERR_TOO_LARGE = 6    /* hla_forward_static: the call's workspace exceeds HLA_STATIC_SCRATCH_BYTES */
} hla_status;

/* I/O element type of Q, K, V, O, dO, dQ, dK, dV and of the feature-map weights.  Accumulation
 * and the key-side state are always fp32 (the paper does not fix a precision). */
typedef enum { HLA_F32 = 0, HLA_BF16 = 1 } hla_dtype;

/* HLA_PHI_MLP : Q and K hold raw head vectors [.., d]; the library applies the feature maps of
 *               App. A.1 (Linear d->d, GELU, Linear d->d_phi, ReLU) — Alg. 1 Step 4.  GELU is the
 *               exact erf form x Phi(x) on the generic path; the MFMA path evaluates a polynomial
 *               fit of it in packed fp16 (|error| <= 5.2e-3 absolute, rms 5e-4 for standard-normal
 *               pre-activations, below the rounding of a bf16 hidden layer), and needs
 *               |pre-activation| < 2.6e5.
 * HLA_PHI_NONE: Q holds phi_q(Q) [.., d_phi] and K holds [phi_k1(K) | ... | phi_kF(K)]
 *               [.., F*d_phi] (factor-major inside the last dim), as the paper's listings for 2
 *               and 3 factors take them.  Features are expected >= 0 (Sec. 4.2); not checked. */
typedef enum { HLA_PHI_MLP = 0, HLA_PHI_NONE = 1 } hla_phi_mode;

/* Which kernels serve the handle.  AUTO picks the MFMA path when the configuration has one: bf16
 * tensors, head_dim 64 or 128, and one of the paper's two forms (App. A.1), F = 3 with d_phi = 6
 * or F = 2 with d_phi = 12. */
typedef enum {
  HLA_PATH_AUTO = 0,
  HLA_PATH_GENERIC = 1, /* fp32 vector-ALU kernels over the literal d_phi^F state; any supported shape */
  HLA_PATH_MFMA = 2     /* bf16 matrix-core kernels; HLA_ERR_UNSUPPORTED if the shape has none */
} hla_kernel_path;

typedef struct {
  int32_t head_dim;      /* d: 32, 64 or 128 (width of V, and of raw Q/K in PHI_MLP mode) */
  int32_t feature_dim;   /* d_phi: paper uses 6 with F=3 and 12 with F=2 (App. A.1) */
  int32_t degree;        /* F, number of Hadamard factors: 1..4; d_phi^F <= 256 */
  float eps;             /* added to eta in the denominator, as in the paper's listings */
  int32_t io_dtype;      /* hla_dtype */
  int32_t phi_mode;      /* hla_phi_mode */
  int32_t kernel_path;   /* hla_kernel_path */
  int32_t max_heads;     /* largest H any call will pass */
  int64_t max_tokens;    /* largest B*N (tokens per head, all batch rows / packed sequences) */
  int32_t max_seqs;      /* largest number of independent sequences (B, or num_seqs when packed) */
  int32_t causal;        /* 0: every token attends to every token of its sequence (the paper's video
                            model); 1: the causal variant of Sec. 4.4, token i attends to tokens
                            j <= i of its sequence (the {0,1} mask; eta_i sums the same entries), which
                            is what the paper's sequential state update C^i = C^{i-1} + T_k,i (x) v_i
                            computes.  Forward and backward on both kernel paths (chunked scans on
                            the MFMA path; on the generic path one workgroup walks a (sequence,
                            head) token tile by token tile: exact in fp32, slow).
                            hla_forward_static returns HLA_ERR_UNSUPPORTED for a causal
                            configuration.  The value modulation of Sec. 4.5 then acts on the
                            causal output. */
  float decay;           /* causal handles only: decay factor lambda of Sec. 4.4.  The paper lets the
                            mask carry decay factors without giving a formula; this library reads it
                            as one scalar lambda in (0, 1] and mask entries lambda^(i-j) for j <= i
                            (state update C^i = lambda C^{i-1} + T_k,i (x) v_i, the normaliser
                            likewise).  0 and 1 both mean no decay.  Anything else than 0 or 1 on a
                            non-causal handle, or a value outside [0, 1], is HLA_ERR_INVALID_ARG. */
} hla_config;

/* Weights of one feature map, device pointers in io_dtype, row-major, applied from the right:
 * h = x W1 + b1 (W1 [d, d]), u = GELU(h) W2 + b2 (W2 [d, d_phi]), phi(x) = max(u, 0).
 * A head stride of 0 shares that array across heads (the default reading of App. A.1: the first
 * layer is sized by the head dimension); otherwise head h's copy starts at ptr + h * stride. */
typedef struct {
  const void* W1;
  const void* b1;
  const void* W2;
  const void* b2;
  int64_t head_stride_W1; /* elements; 0 = shared across heads */
  int64_t head_stride_b1;
  int64_t head_stride_W2;
  int64_t head_stride_b2;
} hla_phi_weights;

/* Strided view of a [B, H, N, width] tensor; the innermost dim is contiguous.  Strides in
 * elements.  The MFMA path additionally needs ptr and all strides 16-byte aligned. */
typedef struct {
  void* ptr;
  int64_t stride_b;
  int64_t stride_h;
  int64_t stride_n;
} hla_tensor;

/* Create a handle and its device workspace (saved features, key-side state, partial sums) on
 * the current HIP device.  Synchronous.  On failure *out is NULL. */
hla_status hla_create(const hla_config* config, hla_handle** out);

/* PHI_MLP only: register the 1+F feature maps in the order phi_q, phi_k1, .., phi_kF.  The
 * library repacks them into its own workspace on `hip_stream`; the caller may free its copies
 * once that stream work has completed.  Must be called again if the weights change. */
hla_status hla_set_phi_weights(hla_handle* h, const hla_phi_weights* maps, int32_t num_maps,
                               void* hip_stream);

/* Forward (Alg. 1 Steps 4-5).  Q, K, V, O are [B, H, N, *] views (widths per phi_mode; V and O
 * are [.., d]).  Dense batch: cu_seqlens = NULL, num_seqs ignored, every batch row is one
 * sequence.  Packed: cu_seqlens is a HOST array of num_seqs+1 non-decreasing token offsets with
 * cu_seqlens[0] = 0 and cu_seqlens[num_seqs] = N, B must be 1; sequence s owns tokens
 * [cu[s], cu[s+1]) and shares no state with the others.  Empty sequences and N = 0 are legal and
 * write nothing.  Keeps the features, the state and the denominators in the handle for a
 * following hla_backward.  Output rows whose eta is 0 are 0/(0+eps) = 0. */
hla_status hla_forward(hla_handle* h, int32_t B, int32_t H, int32_t N, const int32_t* cu_seqlens,
                       int32_t num_seqs, hla_tensor Q, hla_tensor K, hla_tensor V, hla_tensor O,
                       void* hip_stream);

/* Backward of L = sum(O * dO) w.r.t. Q, K, V (the paper relies on autograd; the formulas follow
 * from Theorem 4.2: g_i = dO_i/den_i, s_i = -<dO_i,o_i>/den_i, dT_q,i = C g_i + s_i z,
 * dC = sum_i T_q,i (x) g_i, dz = sum_i s_i T_q,i, dT_k,j = dC v_j + dz, dv_j = dC^T T_k,j, then the
 * chain rule through the outer products and, in PHI_MLP mode, the feature maps; dK sums the F
 * key maps).  Must follow an hla_forward on the same handle with the same B, H, N, cu_seqlens,
 * Q, K, V (HLA_ERR_STATE otherwise); O is that forward's output.  dQ, dK, dV have the shapes of
 * Q, K, V and are fully overwritten. */
hla_status hla_backward(hla_handle* h, int32_t B, int32_t H, int32_t N, const int32_t* cu_seqlens,
                        int32_t num_seqs, hla_tensor Q, hla_tensor K, hla_tensor V, hla_tensor O,
                        hla_tensor dO, hla_tensor dQ, hla_tensor dK, hla_tensor dV,
                        void* hip_stream);

/* Optional outputs of hla_backward, PHI_MLP only: gradients of L = sum(O * dO) w.r.t. the weights
 * of the 1+F feature maps (App. A.1 layers; the paper trains them, Sec. 5, and leaves the
 * formulas to autograd): with du = d(feature) where the ReLU was open, dg = du W2^T,
 * dh = dg * GELU'(h):  dW2 = GELU(h)^T du, db2 = sum du, dW1 = x^T dh, db1 = sum dh, summed over
 * every batch row, sequence and token that uses the map (and over heads when the weights are
 * shared).  DEVICE pointers to fp32 arrays owned by the caller, shaped and ordered like the
 * weights (dW1 [d, d], db1 [d], dW2 [d, d_phi], db2 [d_phi], row-major); accumulation and the
 * results are fp32 whatever io_dtype is.  If the weights were registered per head (any non-zero
 * head stride) each array holds max_heads consecutive copies, head h at ptr + h * (elements of one
 * copy), and a call with H < max_heads leaves the copies of heads >= H untouched. */
typedef struct {
  float* dW1;
  float* db1;
  float* dW2;
  float* db2;
} hla_phi_weight_grads;

/* Register (maps != NULL, num_maps = 1+F, order phi_q, phi_k1, .., phi_kF) or clear (maps = NULL)
 * the weight-gradient outputs.  While registered, every hla_backward OVERWRITES them on its
 * stream after the input gradients; they must stay valid until that work has completed.  Needs a
 * prior hla_set_phi_weights (HLA_ERR_STATE otherwise); registering new weights keeps the outputs
 * unless it switches between shared and per-head weights, which clears them.  A backward over
 * no tokens writes zeros.  d_phi above 16 is HLA_ERR_UNSUPPORTED.
 * The first registration allocates the partial-sum workspace (synchronous; HLA_ERR_ALLOC on
 * failure). */
hla_status hla_set_phi_weight_grads(hla_handle* h, const hla_phi_weight_grads* maps,
                                    int32_t num_maps);

/* Value modulation (Sec. 4.5): with T the normalised attention output of the operator,
 *     O = T + phi_v1(T) * phi_v2(V)          (elementwise product, per token and head)
 * phi_v (App. A.1): h = x W1 + b1 (W1 [d, d]), u = GELU(h) W2 + b2 (W2 [d, d]),
 * phi_v(x) = LayerNorm(u) * gamma + beta over the d channels (biased variance, ln_eps inside the
 * square root).  The paper requires a LayerNorm in phi_v but its figure of the network is missing
 * from the text: this library places it on the output of the second layer.  No ReLU.  The two
 * maps are shared by all heads.  DEVICE pointers in io_dtype, row-major, applied from the right;
 * the library converts them into its own workspace on `hip_stream`.
 *
 * maps = {phi_v1, phi_v2} switches the modulation on for the handle, maps = NULL off.  While on:
 * hla_forward writes the modulated O and keeps T in the handle; hla_backward takes dO as the
 * gradient w.r.t. the modulated O, carries it back through the modulation first (dV receives the
 * share that reaches V through phi_v2 as well) and must follow a forward made in the same mode.
 * The first registration allocates three [max_heads * max_tokens, d] arrays and, on the
 * matrix-core path, 512 bytes per token-head that the forward keeps for the backward (the maps'
 * normalised outputs) (synchronous; HLA_ERR_ALLOC on failure).  Gradients of the modulation's own
 * weights: see hla_set_value_modulation_grads. */
typedef struct {
  const void* W1;
  const void* b1;
  const void* W2;
  const void* b2;
  const void* gamma;
  const void* beta;
} hla_vmod_weights;
hla_status hla_set_value_modulation(hla_handle* h, const hla_vmod_weights* maps, float ln_eps,
                                    void* hip_stream);

/* Optional outputs of hla_backward: gradients of the loss w.r.t. the weights of the two
 * value-modulation maps (App. A.1, Sec. 4.5), summed over every token of every head and batch row
 * (the maps are shared by all of them).  DEVICE pointers to fp32 arrays, caller-owned, shaped like
 * the weights: dW1 [d, d], db1 [d], dW2 [d, d], db2 [d], dgamma [d], dbeta [d].
 *
 * maps = {phi_v1, phi_v2} registers them, maps = NULL clears the registration.  While registered,
 * every hla_backward OVERWRITES them on its stream; they must stay valid until that work has
 * completed.  Needs the modulation switched on (HLA_ERR_STATE otherwise); switching it off clears
 * the registration.  A backward over no tokens writes zeros.  Head dims other than 32, 64, 128 are
 * HLA_ERR_UNSUPPORTED.  The first registration allocates the workspace (per-token factors, 20
 * bytes per token-head and channel, and the partial sums; synchronous; HLA_ERR_ALLOC on
 * failure). */
typedef struct {
  float* dW1;
  float* db1;
  float* dW2;
  float* db2;
  float* dgamma;
  float* dbeta;
} hla_vmod_weight_grads;
hla_status hla_set_value_modulation_grads(hla_handle* h, const hla_vmod_weight_grads* maps);

/* hla_forward for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  No handle: the workspace (features, chunk
 * partial states, the reduced state, token tables) lives in a static device array of
 * HLA_STATIC_SCRATCH_BYTES inside the library, one copy per GPU, held until the process ends.  The
 * call allocates nothing on the device, copies nothing from the host and never synchronises; it
 * runs the same kernels as hla_forward and returns the same bits.
 *   - HLA_PHI_NONE only (Q and K hold features, see hla_phi_mode); dense batches only (every
 *     batch row one sequence).  config->max_heads / max_tokens / max_seqs are ignored: the
 *     workspace is laid out for exactly (B, H, N).
 *   - HLA_ERR_TOO_LARGE if that layout needs more than HLA_STATIC_SCRATCH_BYTES (about 2e5
 *     token-heads B*H*N for the three-factor form at head_dim 128); outputs are then untouched.
 *   - All calls on one GPU share the array and it keeps the last call's contents: calls that
 *     overlap on one GPU (two streams, two threads) race.  Calls on one stream are ordered. */
#define HLA_STATIC_SCRATCH_BYTES (32u << 20)
hla_status hla_forward_static(const hla_config* config, int32_t B, int32_t H, int32_t N, hla_tensor Q,
                              hla_tensor K, hla_tensor V, hla_tensor O, void* hip_stream);

/* Release the workspace.  Synchronises the device first.  NULL is accepted. */
hla_status hla_destroy(hla_handle* h);

/* Static, human-readable name of a status code. */
const char* hla_status_string(hla_status s);

/* Which path serves the handle: HLA_PATH_GENERIC or HLA_PATH_MFMA (never AUTO); -1 for NULL. */
int32_t hla_active_path(const hla_handle* h);

/* ---- Test and bench aids (not part of the operator's interface) ------------------------------- */

/* Intermediate results of the last forward / backward, for tests of the individual steps:
 *   HLA_WS_FEATURES      [B*H*N][(1+F)*d_phi] fp32: phi_q, then phi_k1..phi_kF of every token-head
 *                        (Alg. 1 Step 4), row index (b*H + h)*N + n
 *   HLA_WS_FEATURE_GRADS same layout: gradient w.r.t. those features (after hla_backward).  With
 *                        HLA_PHI_MLP on the MFMA path it is the gradient at the input of the
 *                        maps' final ReLU: entries whose feature is zero hold zero
 *   HLA_WS_DENOMINATORS  [B*H*N] fp32: eta + eps (Sec. 4.2 normaliser)
 * Copies `count` floats to the HOST buffer `host_dst` after synchronising `hip_stream`.  count
 * above what the last call produced is HLA_ERR_INVALID_ARG. */
typedef enum { HLA_WS_FEATURES = 0, HLA_WS_FEATURE_GRADS = 1, HLA_WS_DENOMINATORS = 2 } hla_workspace_kind;
hla_status hla_read_workspace(hla_handle* h, int32_t kind, float* host_dst, int64_t count,
                              void* hip_stream);

/* Per-kernel timing for bench harnesses.  While enabled, every kernel the handle launches is
 * bracketed by a pair of HIP events on the caller's stream.  Enabling (or re-enabling) clears the
 * accumulated records; at most HLA_PROFILE_MAX_RECORDS launches are recorded, later ones run
 * untimed. */
#define HLA_PROFILE_MAX_RECORDS 8192
hla_status hla_profile_enable(hla_handle* h, int32_t on);

/* Synchronises on the recorded events, then reports per distinct kernel: its name (static
 * string), the summed duration in milliseconds and the number of launches.  Writes at most `cap`
 * entries to each non-NULL HOST array and returns the number of distinct kernels recorded. */
int32_t hla_profile_read(hla_handle* h, int32_t cap, const char** names, double* total_ms,
                         int64_t* launches);

#ifdef __cplusplus
}
#endif
#endif /* HLA_H_ */
