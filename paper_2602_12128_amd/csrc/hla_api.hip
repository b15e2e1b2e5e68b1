// C-ABI entry points of libhla: argument validation, workspace ownership, token tables, path
// dispatch and per-kernel event timing.  No arithmetic of the method lives here.
#include <algorithm>
#include <cstring>
#include <new>

#include "hla_handle.h"

// Workspace of hla_forward_static: one copy per GPU, for as long as the process lives.  In host
// code this name is only a handle for hipGetSymbolAddress; the address kernels and fills use is
// the one that call returns, kept per device in g_static below.
static __device__ __align__(256) unsigned char scratch[HLA_STATIC_SCRATCH_BYTES];

namespace hla {

// ---- profiler ---------------------------------------------------------------------------------
const char* Profiler::begin(const char* name, hipStream_t s) {
  if (!on || n_used >= static_cast<size_t>(HLA_PROFILE_MAX_RECORDS)) return nullptr;
  if (n_used == records.size()) {
    ProfileRecord r{name, nullptr, nullptr};
    if (hipEventCreate(&r.start) != hipSuccess) return nullptr;
    if (hipEventCreate(&r.stop) != hipSuccess) {
      (void)hipEventDestroy(r.start);
      return nullptr;
    }
    records.push_back(r);
  }
  records[n_used].name = name;
  (void)hipEventRecord(records[n_used].start, s);
  pending = true;
  return name;
}
void Profiler::end(hipStream_t s) {
  if (!pending) return;
  (void)hipEventRecord(records[n_used].stop, s);
  ++n_used;
  pending = false;
}
void Profiler::clear_records() {
  n_used = 0;
  pending = false;
}
void Profiler::destroy() {
  for (auto& r : records) {
    (void)hipEventDestroy(r.start);
    (void)hipEventDestroy(r.stop);
  }
  records.clear();
  n_used = 0;
}

// ---- token tables -----------------------------------------------------------------------------
static void build_table_host(const hla_handle* hd, int32_t bs, std::vector<BlockEnt>* ents,
                             std::vector<int32_t>* seq_off) {
  const int nseq = static_cast<int>(hd->cu_host.size()) - 1;
  ents->clear();
  seq_off->assign(nseq + 1, 0);
  for (int s = 0; s < nseq; ++s) {
    (*seq_off)[s] = static_cast<int32_t>(ents->size());
    const int32_t lo = hd->cu_host[s], hi = hd->cu_host[s + 1];
    for (int32_t t0 = lo; t0 < hi; t0 += bs) ents->push_back(BlockEnt{0, s, t0, std::min(t0 + bs, hi)});
  }
  (*seq_off)[nseq] = static_cast<int32_t>(ents->size());
}

// Dense batch: batch row s is sequence s, cut into ceil(N / bs) runs.  Built on the device, so a
// call with a shape not seen before copies nothing from the host.
__global__ void k_fill_table_dense(BlockEnt* __restrict__ ents, int32_t* __restrict__ seq_off, int B,
                                   int N, int bs) {
  const int per = (N + bs - 1) / bs;
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < B * per) {
    const int s = i / per, t0 = (i % per) * bs;
    ents[i] = BlockEnt{s, s, t0, t0 + bs < N ? t0 + bs : N};
  }
  if (i <= B) seq_off[i] = i * per;
}

hla_status get_table(hla_handle* hd, int role, int32_t block_tokens, hipStream_t s, hla_token_table** out) {
  if (role < 0 || role >= kTableRoles) return HLA_ERR_INVALID_ARG;
  hla_token_table& t = hd->tables[role];
  if (t.dev == nullptr || block_tokens < t.min_block) return HLA_ERR_INVALID_ARG;
  if (t.block_tokens != block_tokens) t.valid = false;
  if (!t.valid) {
    if (!hd->sig_packed) {
      const int64_t per = (static_cast<int64_t>(hd->sig_N) + block_tokens - 1) / block_tokens;
      const int64_t count = per * hd->sig_B;
      if (count > t.capacity) return HLA_ERR_INVALID_ARG;
      const int64_t threads = std::max<int64_t>(count, hd->sig_B + 1);
      k_fill_table_dense<<<dim3(static_cast<unsigned>((threads + 255) / 256)), dim3(256), 0, s>>>(
          t.dev, t.seq_off_dev, hd->sig_B, hd->sig_N, block_tokens);
      if (hipGetLastError() != hipSuccess) return HLA_ERR_HIP;
      t.count = static_cast<int32_t>(count);
    } else {
      std::vector<BlockEnt> ents;
      std::vector<int32_t> seq_off;
      build_table_host(hd, block_tokens, &ents, &seq_off);
      if (static_cast<int64_t>(ents.size()) > t.capacity) return HLA_ERR_INVALID_ARG;
      // pageable source: the runtime stages it before returning, so the vectors may die here
      if (!ents.empty())
        HLA_HIP_TRY(hipMemcpyAsync(t.dev, ents.data(), ents.size() * sizeof(BlockEnt),
                                   hipMemcpyHostToDevice, s));
      HLA_HIP_TRY(hipMemcpyAsync(t.seq_off_dev, seq_off.data(), seq_off.size() * sizeof(int32_t),
                                 hipMemcpyHostToDevice, s));
      t.count = static_cast<int32_t>(ents.size());
    }
    t.block_tokens = block_tokens;
    t.valid = true;
  }
  *out = &t;
  return HLA_OK;
}

}  // namespace hla

using namespace hla;

namespace {

// Where a handle's device workspace comes from: hipMalloc (one allocation per array, owned by the
// handle), or consecutive 256-byte aligned pieces of a block of device memory that is not the
// handle's (base != nullptr; nothing is allocated and nothing will be freed).
struct Arena {
  unsigned char* base = nullptr;
  size_t cap = 0;
  size_t used = 0;
  template <typename T>
  hla_status alloc(T** p, size_t count) {
    *p = nullptr;
    if (count == 0) count = 1;
    const size_t bytes = count * sizeof(T);
    if (base == nullptr)
      return hipMalloc(reinterpret_cast<void**>(p), bytes) == hipSuccess ? HLA_OK : HLA_ERR_ALLOC;
    const size_t at = (used + 255) / 256 * 256;
    if (at + bytes > cap) return HLA_ERR_TOO_LARGE;
    *p = reinterpret_cast<T*>(base + at);
    used = at + bytes;
    return HLA_OK;
  }
};

void free_all(hla_handle* hd) {
  if (!hd->borrowed_ws) {
    (void)hipFree(hd->feat);
    (void)hipFree(hd->dfeat);
    (void)hipFree(hd->den);
    (void)hipFree(hd->yhat);
    (void)hipFree(hd->state);
    (void)hipFree(hd->dstate);
    (void)hipFree(hd->partial);
    (void)hipFree(hd->path_ws);
    (void)hipFree(hd->w_f32);
    (void)hipFree(hd->wg_partial);
    (void)hipFree(hd->vmod_w);
    (void)hipFree(hd->vmod_wpk);
    (void)hipFree(hd->vmod_wg_partial);
    (void)hipFree(hd->vmod_wg_rows);
    (void)hipFree(hd->vmod_T);
    (void)hipFree(hd->vmod_dT);
    (void)hipFree(hd->vmod_dV);
    for (hla_token_table& t : hd->tables) {
      (void)hipFree(t.dev);
      (void)hipFree(t.seq_off_dev);
    }
  }
  hd->prof.destroy();
}

int64_t ipow(int64_t b, int e) {
  int64_t r = 1;
  for (int i = 0; i < e; ++i) r *= b;
  return r;
}

// Validates the shape arguments shared by forward and backward and refreshes the table signature.
hla_status prepare_call(hla_handle* hd, int32_t B, int32_t H, int32_t N, const int32_t* cu,
                        int32_t num_seqs, bool* empty, int32_t* nseq_eff) {
  if (hd == nullptr) return HLA_ERR_INVALID_ARG;
  if (B < 0 || H < 0 || N < 0) return HLA_ERR_INVALID_ARG;
  const bool packed = cu != nullptr;
  if (packed) {
    if (B != 1 || num_seqs < 0) return HLA_ERR_INVALID_ARG;
    if (cu[0] != 0 || cu[num_seqs] != N) return HLA_ERR_INVALID_ARG;
    for (int s = 0; s < num_seqs; ++s)
      if (cu[s + 1] < cu[s]) return HLA_ERR_INVALID_ARG;
  }
  const int32_t nseq = packed ? num_seqs : B;
  *nseq_eff = nseq;
  *empty = (B == 0 || H == 0 || N == 0 || nseq == 0);
  if (H > hd->cfg.max_heads || nseq > hd->cfg.max_seqs ||
      static_cast<int64_t>(B) * N > hd->cfg.max_tokens)
    return HLA_ERR_INVALID_ARG;
  // table signature
  bool same = hd->sig_B == B && hd->sig_N == N && hd->sig_packed == packed;
  if (same && packed) {
    same = static_cast<int32_t>(hd->cu_host.size()) == num_seqs + 1 &&
           std::memcmp(hd->cu_host.data(), cu, sizeof(int32_t) * (num_seqs + 1)) == 0;
  }
  if (!same) {
    hd->sig_B = B;
    hd->sig_N = N;
    hd->sig_packed = packed;
    if (packed) {
      hd->cu_host.assign(cu, cu + num_seqs + 1);
    } else {
      hd->cu_host.assign(static_cast<size_t>(B) + 1, 0);
    }
    for (hla_token_table& t : hd->tables) t.valid = false;
  }
  hd->g.B = B;
  hd->g.H = H;
  hd->g.N = N;
  return HLA_OK;
}

hla_status validate_config(const hla_config* c) {
  if (c == nullptr) return HLA_ERR_INVALID_ARG;
  if (c->max_heads <= 0 || c->max_tokens <= 0 || c->max_seqs <= 0) return HLA_ERR_INVALID_ARG;
  if (c->io_dtype != HLA_F32 && c->io_dtype != HLA_BF16) return HLA_ERR_INVALID_ARG;
  if (c->phi_mode != HLA_PHI_MLP && c->phi_mode != HLA_PHI_NONE) return HLA_ERR_INVALID_ARG;
  if (c->kernel_path < HLA_PATH_AUTO || c->kernel_path > HLA_PATH_MFMA) return HLA_ERR_INVALID_ARG;
  if (!(c->eps >= 0.0f)) return HLA_ERR_INVALID_ARG;
  if (c->causal != 0 && c->causal != 1) return HLA_ERR_INVALID_ARG;
  if (!(c->decay >= 0.0f && c->decay <= 1.0f)) return HLA_ERR_INVALID_ARG;
  if (!c->causal && c->decay != 0.0f && c->decay != 1.0f) return HLA_ERR_INVALID_ARG;
  if (c->head_dim != 32 && c->head_dim != 64 && c->head_dim != 128) return HLA_ERR_UNSUPPORTED;
  if (c->degree < 1 || c->degree > 4 || c->feature_dim < 1) return HLA_ERR_UNSUPPORTED;
  if (c->feature_dim > 256 || ipow(c->feature_dim, c->degree) > 256) return HLA_ERR_UNSUPPORTED;
  if (static_cast<int64_t>(c->max_heads) * c->max_tokens >= (1ll << 31)) return HLA_ERR_UNSUPPORTED;
  return HLA_OK;
}

// Geometry, kernel path and workspace sizes of a handle for a validated configuration (host only).
hla_status plan_handle(hla_handle* hd, const hla_config& c) {
  hd->cfg = c;
  hd->g = Geom{};
  hd->g.d = c.head_dim;
  hd->g.dphi = c.feature_dim;
  hd->g.F = c.degree;
  hd->g.D = static_cast<int32_t>(ipow(c.feature_dim, c.degree));
  hd->g.nfeat = (1 + c.degree) * c.feature_dim;
  hd->g.eps = c.eps;
  hd->max_th = static_cast<int64_t>(c.max_heads) * c.max_tokens;
  hd->max_units = c.max_seqs * c.max_heads;
  const bool mfma_ok = mfma_supported(c);
  if (c.kernel_path == HLA_PATH_MFMA && !mfma_ok) return HLA_ERR_UNSUPPORTED;
  hd->path = (c.kernel_path == HLA_PATH_GENERIC || !mfma_ok) ? HLA_PATH_GENERIC : HLA_PATH_MFMA;
  hd->g.feat_tiled = hd->path == HLA_PATH_MFMA ? 1 : 0;
  for (hla_token_table& t : hd->tables) t = hla_token_table{};
  return hd->path == HLA_PATH_MFMA ? mfma_workspace_plan(hd) : generic_workspace_plan(hd);
}

// The device arrays the plan asked for.  forward_only leaves out what only a backward touches
// (feature gradients, the state gradient, the generic path's per-token scratch).
hla_status allocate_workspace(hla_handle* hd, Arena& arena, bool forward_only) {
  const hla_config& c = hd->cfg;
  const int64_t feat_rows = (hd->max_th + 31) / 32 * 32;  // whole 32-token groups for the tiled layout
  HLA_TRY(arena.alloc(&hd->feat, feat_rows * hd->g.nfeat));
  if (!forward_only) HLA_TRY(arena.alloc(&hd->dfeat, feat_rows * hd->g.nfeat));
  HLA_TRY(arena.alloc(&hd->den, hd->max_th));
  if (!forward_only) HLA_TRY(arena.alloc(&hd->yhat, hd->yhat_floats));
  HLA_TRY(arena.alloc(&hd->state, hd->max_units * hd->state_stride));
  if (!forward_only) HLA_TRY(arena.alloc(&hd->dstate, hd->max_units * hd->state_stride));
  HLA_TRY(arena.alloc(&hd->partial, hd->max_chunks * c.max_heads * hd->state_stride));
  if (hd->path_ws_bytes > 0) {
    char* p = nullptr;
    HLA_TRY(arena.alloc(&p, hd->path_ws_bytes));
    hd->path_ws = p;
  }
  if (c.phi_mode == HLA_PHI_MLP) {
    const int64_t per_map = static_cast<int64_t>(c.head_dim) * c.head_dim + c.head_dim +
                            static_cast<int64_t>(c.head_dim) * c.feature_dim + c.feature_dim;
    HLA_TRY(arena.alloc(&hd->w_f32, per_map * (1 + c.degree) * c.max_heads));
  }
  for (hla_token_table& t : hd->tables) {
    if (t.min_block <= 0) continue;
    t.capacity = (c.max_tokens + t.min_block - 1) / t.min_block + c.max_seqs;
    HLA_TRY(arena.alloc(&t.dev, t.capacity));
    HLA_TRY(arena.alloc(&t.seq_off_dev, c.max_seqs + 1));
  }
  return HLA_OK;
}

bool bad_view(const hla_tensor& t) { return t.ptr == nullptr; }

}  // namespace

extern "C" {

const char* hla_status_string(hla_status s) {
  switch (s) {
    case HLA_OK: return "HLA_OK";
    case HLA_ERR_INVALID_ARG: return "HLA_ERR_INVALID_ARG";
    case HLA_ERR_UNSUPPORTED: return "HLA_ERR_UNSUPPORTED";
    case HLA_ERR_ALLOC: return "HLA_ERR_ALLOC";
    case HLA_ERR_HIP: return "HLA_ERR_HIP";
    case HLA_ERR_STATE: return "HLA_ERR_STATE";
    case HLA_ERR_TOO_LARGE: return "HLA_ERR_TOO_LARGE";
  }
  return "HLA_ERR_UNKNOWN";
}

hla_status hla_create(const hla_config* c, hla_handle** out) {
  if (out == nullptr) return HLA_ERR_INVALID_ARG;
  *out = nullptr;
  HLA_TRY(validate_config(c));
  hla_handle* hd = new (std::nothrow) hla_handle();
  if (hd == nullptr) return HLA_ERR_ALLOC;
  hla_status st = plan_handle(hd, *c);
  if (st != HLA_OK) {  // nothing on the device yet
    delete hd;
    return st;
  }
  Arena arena;  // hipMalloc
  st = allocate_workspace(hd, arena, /*forward_only=*/false);
  // padding entries of packed operands are never written afterwards and must read as zero
  if (st == HLA_OK && hd->path_ws_bytes > 0 && hipMemset(hd->path_ws, 0, hd->path_ws_bytes) != hipSuccess)
    st = HLA_ERR_HIP;
  if (st == HLA_OK) st = hd->path == HLA_PATH_MFMA ? mfma_prepare_kernels(hd) : generic_prepare_kernels(hd);
  if (st == HLA_OK && hipDeviceSynchronize() != hipSuccess) st = HLA_ERR_HIP;
  if (st != HLA_OK) {
    free_all(hd);
    delete hd;
    return st;
  }
  *out = hd;
  return HLA_OK;
}

hla_status hla_destroy(hla_handle* hd) {
  if (hd == nullptr) return HLA_OK;
  (void)hipDeviceSynchronize();
  free_all(hd);
  delete hd;
  return HLA_OK;
}

int32_t hla_active_path(const hla_handle* hd) { return hd == nullptr ? -1 : hd->path; }

hla_status hla_set_phi_weights(hla_handle* hd, const hla_phi_weights* maps, int32_t num_maps,
                               void* hip_stream) {
  if (hd == nullptr || maps == nullptr) return HLA_ERR_INVALID_ARG;
  if (hd->cfg.phi_mode != HLA_PHI_MLP) return HLA_ERR_STATE;
  if (num_maps != 1 + hd->cfg.degree) return HLA_ERR_INVALID_ARG;
  for (int m = 0; m < num_maps; ++m)
    if (!maps[m].W1 || !maps[m].b1 || !maps[m].W2 || !maps[m].b2) return HLA_ERR_INVALID_ARG;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const int32_t heads_w_before = hd->have_weights ? hd->phi.heads_w : 0;
  HLA_TRY(convert_weights_to_f32(hd, maps, s));
  // gradient arrays registered for the other sharing mode no longer have the right shape
  if (heads_w_before != 0 && heads_w_before != hd->phi.heads_w) hd->wg_on = false;
  HLA_TRY(hd->path == HLA_PATH_MFMA ? mfma_set_weights(hd, s) : generic_set_weights(hd, s));
  hd->have_weights = true;
  hd->have_forward = false;
  return HLA_OK;
}

hla_status hla_set_phi_weight_grads(hla_handle* hd, const hla_phi_weight_grads* maps,
                                    int32_t num_maps) {
  if (hd == nullptr) return HLA_ERR_INVALID_ARG;
  if (hd->cfg.phi_mode != HLA_PHI_MLP) return HLA_ERR_STATE;
  if (maps == nullptr) {
    hd->wg_on = false;
    return HLA_OK;
  }
  if (!hd->have_weights) return HLA_ERR_STATE;
  if (num_maps != 1 + hd->cfg.degree) return HLA_ERR_INVALID_ARG;
  for (int m = 0; m < num_maps; ++m)
    if (!maps[m].dW1 || !maps[m].db1 || !maps[m].dW2 || !maps[m].db2) return HLA_ERR_INVALID_ARG;
  if (hd->cfg.feature_dim > 16) return HLA_ERR_UNSUPPORTED;  // the kernels keep a W2 row in 16 registers
  if (hd->wg_partial == nullptr) {
    const Geom& g = hd->g;
    hd->wg_part_floats = static_cast<int64_t>(g.d) * g.d + g.d + static_cast<int64_t>(g.d) * g.dphi + g.dphi;
    // one partial sum per wave group of a grid of at most 256 workgroups (eight waves, a group per
    // d / 32 hidden blocks: two groups at d = 128, four at d = 64), and never fewer than one per
    // (map, head)
    const int64_t groups = g.d >= 32 ? 8 * 32 / g.d : 8;
    hd->wg_parts_cap = 256 * (groups < 2 ? 2 : groups) + 2 * static_cast<int64_t>(num_maps) * hd->cfg.max_heads;
    Arena arena;  // hipMalloc
    HLA_TRY(arena.alloc(&hd->wg_partial, hd->wg_parts_cap * hd->wg_part_floats));
  }
  for (int m = 0; m < num_maps; ++m) hd->wg_out[m] = maps[m];
  hd->wg_on = true;
  return HLA_OK;
}

hla_status hla_set_value_modulation(hla_handle* hd, const hla_vmod_weights* maps, float ln_eps,
                                    void* hip_stream) {
  if (hd == nullptr) return HLA_ERR_INVALID_ARG;
  hd->have_forward = false;
  if (maps == nullptr) {
    hd->vmod_on = false;
    hd->vmod_wg_on = false;
    return HLA_OK;
  }
  if (!(ln_eps >= 0.0f)) return HLA_ERR_INVALID_ARG;
  for (int m = 0; m < 2; ++m)
    if (!maps[m].W1 || !maps[m].b1 || !maps[m].W2 || !maps[m].b2 || !maps[m].gamma || !maps[m].beta)
      return HLA_ERR_INVALID_ARG;
  if (hd->borrowed_ws) return HLA_ERR_STATE;
  if (hd->vmod_w == nullptr) {
    const int64_t d = hd->g.d;
    const size_t elem = hd->cfg.io_dtype == HLA_F32 ? 4 : 2;
    Arena arena;  // hipMalloc
    char *t = nullptr, *dt = nullptr, *dv = nullptr;
    hla_status st = arena.alloc(&hd->vmod_w, 2 * (4 * d * d + 4 * d));
    if (st == HLA_OK) st = arena.alloc(&t, static_cast<size_t>(hd->max_th) * d * elem);
    if (st == HLA_OK) st = arena.alloc(&dt, static_cast<size_t>(hd->max_th) * d * elem);
    if (st == HLA_OK) st = arena.alloc(&dv, static_cast<size_t>(hd->max_th) * d * elem);
    unsigned char* wpk = nullptr;
    if (st == HLA_OK && vmod_mfma_supported(hd)) {
      st = arena.alloc(&wpk, vmod_mfma_workspace_bytes(hd));
      if (st == HLA_OK) st = vmod_mfma_prepare_kernels(hd);
    }
    if (st != HLA_OK) {
      (void)hipFree(hd->vmod_w);
      (void)hipFree(wpk);
      (void)hipFree(t);
      (void)hipFree(dt);
      (void)hipFree(dv);
      hd->vmod_w = nullptr;
      return st;
    }
    hd->vmod_wpk = wpk;
    hd->vmod_T = t;
    hd->vmod_dT = dt;
    hd->vmod_dV = dv;
  }
  HLA_TRY(vmod_set_weights(hd, maps, static_cast<hipStream_t>(hip_stream)));
  hd->vmod_ln_eps = ln_eps;
  hd->vmod_on = true;
  return HLA_OK;
}

hla_status hla_set_value_modulation_grads(hla_handle* hd, const hla_vmod_weight_grads* maps) {
  if (hd == nullptr) return HLA_ERR_INVALID_ARG;
  if (maps == nullptr) {
    hd->vmod_wg_on = false;
    return HLA_OK;
  }
  if (!hd->vmod_on) return HLA_ERR_STATE;
  const int d = hd->g.d;
  if (d != 32 && d != 64 && d != 128) return HLA_ERR_UNSUPPORTED;
  for (int m = 0; m < 2; ++m)
    if (!maps[m].dW1 || !maps[m].db1 || !maps[m].dW2 || !maps[m].db2 || !maps[m].dgamma || !maps[m].dbeta)
      return HLA_ERR_INVALID_ARG;
  if (hd->vmod_wg_partial == nullptr) {
    Arena arena;  // hipMalloc
    float *part = nullptr, *rows = nullptr;
    size_t part_floats = static_cast<size_t>(kVmodWgradParts) * vmod_wgrad_part_floats(d);
    size_t row_floats = static_cast<size_t>(3) * hd->max_th * d;
    if (hd->vmod_wpk != nullptr) {  // matrix-core handles: ten bf16 factor arrays, per-wave partials
      part_floats = std::max(part_floats, static_cast<size_t>(vmod_mfma_partial_floats(hd)));
      row_floats = std::max(row_floats, static_cast<size_t>(vmod_mfma_factor_floats(hd)));
    }
    hla_status st = arena.alloc(&part, part_floats);
    if (st == HLA_OK) st = arena.alloc(&rows, row_floats);
    if (st != HLA_OK) {
      (void)hipFree(part);
      (void)hipFree(rows);
      return st;
    }
    hd->vmod_wg_partial = part;
    hd->vmod_wg_rows = rows;
  }
  for (int m = 0; m < 2; ++m) hd->vmod_wg_out[m] = maps[m];
  hd->vmod_wg_on = true;
  return HLA_OK;
}

hla_status hla_forward(hla_handle* hd, int32_t B, int32_t H, int32_t N, const int32_t* cu_seqlens,
                       int32_t num_seqs, hla_tensor Q, hla_tensor K, hla_tensor V, hla_tensor O,
                       void* hip_stream) {
  bool empty = false;
  int32_t nseq = 0;
  HLA_TRY(prepare_call(hd, B, H, N, cu_seqlens, num_seqs, &empty, &nseq));
  hd->have_forward = false;
  if (hd->cfg.phi_mode == HLA_PHI_MLP && !hd->have_weights) return HLA_ERR_STATE;
  if (!empty && (bad_view(Q) || bad_view(K) || bad_view(V) || bad_view(O)))
    return HLA_ERR_INVALID_ARG;
  hla_call_args a{};
  a.B = B;
  a.H = H;
  a.N = N;
  a.num_seqs = nseq;
  a.packed = cu_seqlens != nullptr;
  a.Q = make_view(Q);
  a.K = make_view(K);
  a.V = make_view(V);
  a.O = make_view(O);
  a.stream = static_cast<hipStream_t>(hip_stream);
  if (!empty) {
    // with value modulation the operator's own output T goes to the handle and the caller's O
    // receives T + phi_v1(T) * phi_v2(V)
    if (hd->vmod_on) a.O = vmod_view(hd->vmod_T, hd->g);
    HLA_TRY(hd->path == HLA_PATH_MFMA ? mfma_forward(hd, a) : generic_forward(hd, a));
    if (hd->vmod_on) {
      a.O = make_view(O);
      HLA_TRY(vmod_forward(hd, a));
    }
  }
  hd->fw_vmod = hd->vmod_on;
  hd->have_forward = true;
  hd->fw_B = B;
  hd->fw_H = H;
  hd->fw_N = N;
  hd->fw_packed = a.packed;
  hd->fw_cu = hd->cu_host;
  hd->fw_Q = Q.ptr;
  hd->fw_K = K.ptr;
  hd->fw_V = V.ptr;
  return HLA_OK;
}

hla_status hla_backward(hla_handle* hd, int32_t B, int32_t H, int32_t N, const int32_t* cu_seqlens,
                        int32_t num_seqs, hla_tensor Q, hla_tensor K, hla_tensor V, hla_tensor O,
                        hla_tensor dO, hla_tensor dQ, hla_tensor dK, hla_tensor dV,
                        void* hip_stream) {
  bool empty = false;
  int32_t nseq = 0;
  if (hd == nullptr) return HLA_ERR_INVALID_ARG;
  // The tables and the saved features belong to the last forward: check before touching them.
  {
    const bool packed = cu_seqlens != nullptr;
    bool same = hd->have_forward && hd->fw_B == B && hd->fw_H == H && hd->fw_N == N &&
                hd->fw_packed == packed && hd->fw_Q == Q.ptr && hd->fw_K == K.ptr &&
                hd->fw_V == V.ptr && hd->fw_vmod == hd->vmod_on;
    if (same && packed) {
      same = num_seqs >= 0 && static_cast<int32_t>(hd->fw_cu.size()) == num_seqs + 1 &&
             std::memcmp(hd->fw_cu.data(), cu_seqlens, sizeof(int32_t) * (num_seqs + 1)) == 0;
    }
    if (!same) return HLA_ERR_STATE;
  }
  HLA_TRY(prepare_call(hd, B, H, N, cu_seqlens, num_seqs, &empty, &nseq));
  if (empty) {
    // no token contributes: the registered weight gradients are still overwritten, with zeros
    if (hd->wg_on && H > 0)
      HLA_TRY(weight_grads_reduce(hd, 0, hd->phi.heads_w == 1 ? 1 : H, 0.0f, 0.0f, 0.0f, 0.0f,
                                  static_cast<hipStream_t>(hip_stream)));
    if (hd->vmod_on && hd->vmod_wg_on) {
      hla_call_args z{};
      z.stream = static_cast<hipStream_t>(hip_stream);
      HLA_TRY(vmod_weight_grads(hd, z, true));
    }
    return HLA_OK;
  }
  if (bad_view(Q) || bad_view(K) || bad_view(V) || bad_view(O) || bad_view(dO) || bad_view(dQ) ||
      bad_view(dK) || bad_view(dV))
    return HLA_ERR_INVALID_ARG;
  hla_call_args a{};
  a.B = B;
  a.H = H;
  a.N = N;
  a.num_seqs = nseq;
  a.packed = cu_seqlens != nullptr;
  a.Q = make_view(Q);
  a.K = make_view(K);
  a.V = make_view(V);
  a.O = make_view(O);
  a.dO = make_view(dO);
  a.dQ = make_view(dQ);
  a.dK = make_view(dK);
  a.dV = make_view(dV);
  a.stream = static_cast<hipStream_t>(hip_stream);
  const hla::View dO_caller = a.dO, O_caller = a.O;
  if (hd->vmod_on) {
    // back through the modulation first: the operator then sees dT as its upstream gradient and
    // T as its output; the modulation's share of dV is added once the operator has written dV
    // (from the caller's dO again), and the modulation's own weight gradients follow that
    HLA_TRY(vmod_backward(hd, a));
    a.dO = vmod_view(hd->vmod_dT, hd->g);
    a.O = vmod_view(hd->vmod_T, hd->g);
  }
  HLA_TRY(hd->path == HLA_PATH_MFMA ? mfma_backward(hd, a) : generic_backward(hd, a));
  if (hd->vmod_on) {
    hla_call_args m = a;
    m.dO = dO_caller;
    m.O = O_caller;
    HLA_TRY(vmod_add_value_grads(hd, m));
    if (hd->vmod_wg_on) HLA_TRY(vmod_weight_grads(hd, m, false));
  }
  if (hd->wg_on) HLA_TRY(phi_weight_grads(hd, a));
  return HLA_OK;
}

// ---- forward without a handle ---------------------------------------------------------------------
namespace {

__global__ void k_fill_zero(uint32_t* __restrict__ p, int64_t words) {
  for (int64_t i = blockIdx.x * static_cast<int64_t>(blockDim.x) + threadIdx.x; i < words;
       i += static_cast<int64_t>(gridDim.x) * blockDim.x)
    p[i] = 0u;
}

constexpr int kMaxDevices = 64;
struct StaticSlot {
  unsigned char* ptr = nullptr;  // device address of this GPU's copy of `scratch`
  hla_handle* hd = nullptr;      // host-side bookkeeping; its device pointers point into `scratch`
  bool planned = false;          // hd is laid out for `cfg`
  hla_config cfg{};
};
StaticSlot g_static[kMaxDevices];

bool same_config(const hla_config& a, const hla_config& b) {
  return a.head_dim == b.head_dim && a.feature_dim == b.feature_dim && a.degree == b.degree &&
         a.eps == b.eps && a.io_dtype == b.io_dtype && a.phi_mode == b.phi_mode &&
         a.kernel_path == b.kernel_path && a.causal == b.causal && a.decay == b.decay && a.max_heads == b.max_heads &&
         a.max_tokens == b.max_tokens && a.max_seqs == b.max_seqs;
}

}  // namespace

hla_status hla_forward_static(const hla_config* config, int32_t B, int32_t H, int32_t N, hla_tensor Q,
                              hla_tensor K, hla_tensor V, hla_tensor O, void* hip_stream) {
  if (config == nullptr || B < 0 || H < 0 || N < 0) return HLA_ERR_INVALID_ARG;
  if (config->phi_mode != HLA_PHI_NONE || config->causal != 0) return HLA_ERR_UNSUPPORTED;
  if (B == 0 || H == 0 || N == 0) return HLA_OK;
  if (bad_view(Q) || bad_view(K) || bad_view(V) || bad_view(O)) return HLA_ERR_INVALID_ARG;
  // the workspace is laid out for exactly this call's sizes
  hla_config c = *config;
  c.max_heads = H;
  c.max_tokens = static_cast<int64_t>(B) * N;
  c.max_seqs = B;
  HLA_TRY(validate_config(&c));
  int dev = -1;
  HLA_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return HLA_ERR_UNSUPPORTED;
  StaticSlot& sl = g_static[dev];
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  if (sl.ptr == nullptr) {  // first call on this device
    void* p = nullptr;
    HLA_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (p == nullptr) return HLA_ERR_HIP;
    hla_handle* hd = new (std::nothrow) hla_handle();
    if (hd == nullptr) return HLA_ERR_ALLOC;
    sl.hd = hd;
    sl.ptr = static_cast<unsigned char*>(p);
  }
  hla_handle* hd = sl.hd;
  if (!sl.planned || !same_config(sl.cfg, c)) {
    sl.planned = false;
    *hd = hla_handle();
    hd->borrowed_ws = true;
    HLA_TRY(plan_handle(hd, c));
    Arena arena;
    arena.base = sl.ptr;
    arena.cap = HLA_STATIC_SCRATCH_BYTES;
    HLA_TRY(allocate_workspace(hd, arena, /*forward_only=*/true));  // HLA_ERR_TOO_LARGE: does not fit
    if (hd->path == HLA_PATH_MFMA) HLA_TRY(mfma_prepare_kernels(hd));
    // the array keeps what the last call left: padding entries of the packed operands must read
    // as zero (a fill kernel rather than a memset node, so that the call can be captured)
    if (hd->path_ws_bytes > 0) {
      const int64_t words = static_cast<int64_t>(hd->path_ws_bytes / 4);
      k_fill_zero<<<dim3(static_cast<unsigned>(std::min<int64_t>((words + 255) / 256, 1024))), dim3(256), 0, s>>>(
          static_cast<uint32_t*>(hd->path_ws), words);
      if (hipGetLastError() != hipSuccess) return HLA_ERR_HIP;
    }
    sl.cfg = c;
    sl.planned = true;
  }
  bool empty = false;
  int32_t nseq = 0;
  HLA_TRY(prepare_call(hd, B, H, N, nullptr, 0, &empty, &nseq));
  hla_call_args a{};
  a.B = B;
  a.H = H;
  a.N = N;
  a.num_seqs = nseq;
  a.packed = false;
  a.Q = make_view(Q);
  a.K = make_view(K);
  a.V = make_view(V);
  a.O = make_view(O);
  a.stream = s;
  return hd->path == HLA_PATH_MFMA ? mfma_forward(hd, a) : generic_forward(hd, a);
}

hla_status hla_read_workspace(hla_handle* hd, int32_t kind, float* host_dst, int64_t count,
                              void* hip_stream) {
  if (hd == nullptr || host_dst == nullptr || count < 0) return HLA_ERR_INVALID_ARG;
  if (!hd->have_forward) return HLA_ERR_STATE;
  const int64_t th = static_cast<int64_t>(hd->fw_B) * hd->fw_H * hd->fw_N;
  const float* src = nullptr;
  int64_t avail = 0;
  switch (kind) {
    case HLA_WS_FEATURES: src = hd->feat; avail = th * hd->g.nfeat; break;
    case HLA_WS_FEATURE_GRADS: src = hd->dfeat; avail = th * hd->g.nfeat; break;
    case HLA_WS_DENOMINATORS: src = hd->den; avail = th; break;
    default: return HLA_ERR_INVALID_ARG;
  }
  if (count > avail) return HLA_ERR_INVALID_ARG;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  HLA_HIP_TRY(hipStreamSynchronize(s));
  if (count == 0) return HLA_OK;
  if (kind != HLA_WS_DENOMINATORS && hd->g.feat_tiled) {
    // the workspace is tiled on the device; hand out the documented [token-head][feature] order
    const int64_t rows = (th + 31) / 32 * 32;
    std::vector<float> raw(static_cast<size_t>(rows * hd->g.nfeat));
    HLA_HIP_TRY(hipMemcpy(raw.data(), src, raw.size() * sizeof(float), hipMemcpyDeviceToHost));
    for (int64_t i = 0; i < count; ++i)
      host_dst[i] = raw[static_cast<size_t>(hd->g.fidx(i / hd->g.nfeat, static_cast<int>(i % hd->g.nfeat)))];
    return HLA_OK;
  }
  HLA_HIP_TRY(hipMemcpy(host_dst, src, count * sizeof(float), hipMemcpyDeviceToHost));
  return HLA_OK;
}

hla_status hla_profile_enable(hla_handle* hd, int32_t on) {
  if (hd == nullptr) return HLA_ERR_INVALID_ARG;
  hd->prof.on = on != 0;
  hd->prof.clear_records();
  return HLA_OK;
}

int32_t hla_profile_read(hla_handle* hd, int32_t cap, const char** names, double* total_ms,
                         int64_t* launches) {
  if (hd == nullptr) return 0;
  std::vector<const char*> uniq;
  std::vector<double> ms;
  std::vector<int64_t> cnt;
  for (size_t i = 0; i < hd->prof.n_used; ++i) {
    ProfileRecord& r = hd->prof.records[i];
    if (hipEventSynchronize(r.stop) != hipSuccess) continue;
    float t = 0.f;
    if (hipEventElapsedTime(&t, r.start, r.stop) != hipSuccess) continue;
    size_t k = 0;
    for (; k < uniq.size(); ++k)
      if (uniq[k] == r.name || std::strcmp(uniq[k], r.name) == 0) break;
    if (k == uniq.size()) {
      uniq.push_back(r.name);
      ms.push_back(0.0);
      cnt.push_back(0);
    }
    ms[k] += t;
    cnt[k] += 1;
  }
  for (size_t k = 0; k < uniq.size() && static_cast<int32_t>(k) < cap; ++k) {
    if (names) names[k] = uniq[k];
    if (total_ms) total_ms[k] = ms[k];
    if (launches) launches[k] = cnt[k];
  }
  return static_cast<int32_t>(uniq.size());
}

}  // extern "C"
