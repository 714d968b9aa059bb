// C ABI of libkvp and the host-side launch plan of the time-to-first-token path
// (Algorithm "KV Prediction Inference", Sec. 4.1): auxiliary prefill -> predictor -> one base
// step over the predicted cache -> greedy first token.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/kvp.h"
#include "common.h"
#include "launch.h"
#include "mfma.h"

using namespace kvp;

namespace {

thread_local char g_err[512] = "";

// Scratch of kvp_generation_step_static: device memory that is part of the library's code object, so a
// caller that may not allocate (HIP graph capture, a serving loop that forbids it) needs no workspace.
// Every GPU the library runs on holds its own copy until the process ends.  In host code the array's
// name is only a handle for hipGetSymbolAddress: the per-device address is looked up once per device in
// kvp_load_weights and kept in g_scratch_ptr; kernels are always given that address, never the name.
static __device__ __align__(256) unsigned char scratch[KVP_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

// Address of the static scratch array on the current device (looked up on first use per device).
hipError_t scratch_address(int device, void** out) {
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
  if (!g_scratch_ptr[device]) {
    void* p = nullptr;
    hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    g_scratch_ptr[device] = p;
  }
  *out = g_scratch_ptr[device];
  return hipSuccess;
}

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

struct ModelW {
  const void* embed = nullptr;
  const void* final_norm = nullptr;
  const void* lm_head = nullptr;
  std::vector<const void*> attn_norm, wq, wk, wv, wo, ffn_norm, w_gate, w_up, w_down;
  std::vector<const void*> q_norm, k_norm;   // optional query / key normalisation gains [head_dim] (all NULL: trait off)
  bool qk_norm() const { return !q_norm.empty() && q_norm[0] != nullptr; }
};

struct ProfEvent {   // one event after each launch (group); cls < 0 marks the start of a run
  hipEvent_t ev;
  int cls;
};

size_t align_up(size_t v) { return (v + 255) & ~size_t(255); }

struct Workspace {   // byte offsets into the caller's workspace
  size_t aux_k, aux_v, x, h, q, attn, gu, act, vt;
  size_t vt_layer;   // bytes of one auxiliary layer's transposed values (0: no matrix-core kernels); vt holds every layer
  size_t y, bq, bk, bv, battn, bact, part, logits, uh, ul, oh, ol, ah, al, ssq;
  size_t qw, rw;     // absorbed step: queries mapped to the auxiliary width, weighted auxiliary values  [B][n_q][Ka]
  size_t total;
  int n_splits;   // decode-attention splits of the widest layer (layers of one width: of every layer)
  int plan_T;     // attention length the splits were planned for
};

struct PlanRegion {   // one carved region of the workspace, for kvp_debug_plan
  const char* name;
  size_t offset, bytes;
};

}  // namespace

struct kvp_handle {
  kvp_config cfg;
  std::vector<int32_t> layer_map;
  ModelW base, aux;
  // widths of every layer (copies of the optional per-layer arrays, else the scalar widths)
  std::vector<int32_t> b_nq, b_nkv, b_f, a_nq, a_nkv, a_f;
  // shape of one layer: the stack's shape with that layer's head counts / feed-forward width
  kvp_model_shape layer_shape(bool is_base, int l) const {
    kvp_model_shape m = is_base ? cfg.base : cfg.aux;
    m.n_q_heads = (is_base ? b_nq : a_nq)[l];
    m.n_kv_heads = (is_base ? b_nkv : a_nkv)[l];
    m.ffn_dim = (is_base ? b_f : a_f)[l];
    m.layer_n_q_heads = m.layer_n_kv_heads = m.layer_ffn_dim = nullptr;
    return m;
  }
  std::vector<const void*> pred_wk, pred_wv;
  size_t esize = 4;
  bool use_mfma = false;      // bf16 MFMA kernels serve this configuration
  bool force_generic = false; // KVP_FORCE_GENERIC=1: shape-generic kernels everywhere (tests)
  float2* rope_aux = nullptr;  // device [max_seq][aux.hd/2]
  float2* rope_base = nullptr; // device [max_seq][base.hd/2]
  void* mfma_tables = nullptr; // device tables of the MFMA predictor
  uint32_t* flags = nullptr;   // device word of KVP_FLAG_* bits set by kernels (kvp_check_flags)
  int pred_main = -1;          // KVP_PRED_MAIN at load time: 0 / 1 force the predictor's stream, -1 = by prompt size
  int device = -1;             // HIP device the handle was loaded on
  // second stream for running the base chain beside the auxiliary chain (see run_overlapped)
  hipStream_t side = nullptr;
  hipEvent_t ev_start = nullptr, ev_done = nullptr;
  std::vector<hipEvent_t> ev_kv;   // [aux.n_layers]: K/V of that auxiliary layer are complete
  bool overlap = false;
  // profiling
  bool prof_on = false;
  std::vector<ProfEvent> prof_pool;
  size_t prof_used = 0;
  double prof_ms[KVP_KC_COUNT] = {};
  int64_t prof_n[KVP_KC_COUNT] = {};
};

namespace {

// The absorbed base step (kernels_absorbed.hip) runs its attention on the matrix cores for these widths
bool absorbed_on_mfma(const kvp_handle* h, int Ka) {
  return h->use_mfma && !h->force_generic && h->cfg.dtype == KVP_DTYPE_BF16 && absorbed_mfma_supported(Ka);
}
int absorbed_splits(const kvp_handle* h, int B, int n_q, int Ka, int T) {
  if (absorbed_on_mfma(h, Ka)) return absorbed_mfma_splits(B, n_q, T);
  return decode_attn_splits(B, n_q >= 4 ? n_q / 4 : 1, T);
}
// Upper bound of absorbed_splits over every prompt length up to T: the matrix-core kernel rounds its chunks to 128 keys,
// so its split count is not monotone in T (8192 keys: 64 chunks of 128; 8208 keys: 33 chunks of 256), and a workspace
// sized for T must also serve shorter prompts.
int absorbed_splits_bound(const kvp_handle* h, int B, int n_q, int Ka, int T) {
  if (!absorbed_on_mfma(h, Ka)) return absorbed_splits(h, B, n_q, Ka, T);   // min(want, ceil(T / 64)): monotone
  const int tiles = (n_q + 15) / 16, want = (512 + B * tiles - 1) / (B * tiles), by_len = (T + 127) / 128;
  return want < by_len ? want : by_len;
}

// Carves the caller's workspace for a B x T call.  base_only: only what one base-model step over
// an existing cache needs (the generation loop) -- no auxiliary cache, no prefill activations, no
// buffers of the absorbed step; T is then the attention length.  `regions` (optional) receives
// every carved region in order.
Workspace plan_workspace(const kvp_handle* h, int B, int T, bool base_only = false, std::vector<PlanRegion>* regions = nullptr) {
  const kvp_config& c = h->cfg;
  size_t N = base_only ? 0 : (size_t)B * T, es = h->esize;
  size_t Ka = (size_t)c.aux.n_kv_heads * c.aux.head_dim, qa = (size_t)c.aux.n_q_heads * c.aux.head_dim;
  size_t qb = (size_t)c.base.n_q_heads * c.base.head_dim;
  Workspace w{};
  size_t off = 0;
  auto take = [&](const char* name, size_t bytes) {
    size_t o = off;
    off = align_up(off + bytes);
    if (regions) regions->push_back(PlanRegion{name, o, bytes});
    return o;
  };
  w.aux_k = take("aux_k", (size_t)c.aux.n_layers * N * Ka * es);
  w.aux_v = take("aux_v", (size_t)c.aux.n_layers * N * Ka * es);
  w.x = take("x", N * c.aux.d_model * sizeof(float));
  w.h = take("h", N * c.aux.d_model * es);
  w.q = take("q", N * qa * es);
  w.attn = take("attn", N * qa * es);
  w.gu = take("gu", h->use_mfma ? 0 : N * 2 * (size_t)c.aux.ffn_dim * es);
  w.act = take("act", N * (size_t)c.aux.ffn_dim * es);
  w.vt_layer = (h->use_mfma && !base_only) ? align_up(mfma_vt_bytes(&c, B, T)) : 0;
  w.vt = take("vt", w.vt_layer * c.aux.n_layers);
  w.y = take("y", (size_t)B * c.base.d_model * sizeof(float));
  w.bq = take("bq", (size_t)B * qb * sizeof(float));
  w.bk = take("bk", (size_t)B * c.base.n_kv_heads * c.base.head_dim * sizeof(float));   // generation step: own key / value
  w.bv = take("bv", (size_t)B * c.base.n_kv_heads * c.base.head_dim * sizeof(float));
  w.battn = take("battn", (size_t)B * qb * sizeof(float));
  w.bact = take("bact", (size_t)B * c.base.ffn_dim * sizeof(float));
  w.n_splits = decode_attn_splits(B, c.base.n_kv_heads, T);
  w.plan_T = T;
  size_t part_elems = 0;                       // layers of different width split differently: size for the largest
  for (int i = 0; i < c.base.n_layers; ++i) {
    size_t e = (size_t)decode_attn_splits(B, h->b_nkv[i], T) * B * h->b_nq[i] * (c.base.head_dim + kPartPad);
    if (e > part_elems) part_elems = e;
    if (base_only) continue;
    const int Ka_i = h->a_nkv[h->layer_map[i]] * c.aux.head_dim;       // the absorbed step's partials are Ka wide
    e = (size_t)absorbed_splits_bound(h, B, h->b_nq[i], Ka_i, T) * B * h->b_nq[i] * (Ka_i + kPartPad);
    if (e > part_elems) part_elems = e;
  }
  w.part = take("part", part_elems * sizeof(float));
  w.qw = take("qw", base_only ? 0 : (size_t)B * c.base.n_q_heads * Ka * sizeof(float));
  w.rw = take("rw", base_only ? 0 : (size_t)B * c.base.n_q_heads * Ka * sizeof(float));
  w.logits = take("logits", (size_t)B * c.vocab * sizeof(float));
  w.uh = take("uh", (size_t)B * c.base.d_model * 2); w.ul = take("ul", (size_t)B * c.base.d_model * 2);
  w.oh = take("oh", (size_t)B * qb * 2); w.ol = take("ol", (size_t)B * qb * 2);
  w.ah = take("ah", (size_t)B * c.base.ffn_dim * 2); w.al = take("al", (size_t)B * c.base.ffn_dim * 2);
  w.ssq = take("ssq", (size_t)B * chain_ssq_parts(c.base.d_model, B) * sizeof(float));
  w.total = off;
  return w;
}

// Per-class timing: ONE event is recorded after each launch (group); the time between two
// consecutive events on the stream is charged to the class of the later one.  A single event
// between kernels perturbs the stream far less than a start/stop pair around every launch.
void prof_mark(kvp_handle* h, hipStream_t s, int cls) {
  if (!h->prof_on) return;
  if (h->prof_used == h->prof_pool.size()) {
    ProfEvent e{};
    if (hipEventCreate(&e.ev) != hipSuccess) return;
    h->prof_pool.push_back(e);
  }
  ProfEvent& e = h->prof_pool[h->prof_used++];
  e.cls = cls;
  (void)hipEventRecord(e.ev, s);
}
struct Timed {
  kvp_handle* h;
  hipStream_t s;
  int cls;
  Timed(kvp_handle* hh, hipStream_t ss, int c) : h(hh), s(ss), cls(c) {}
  ~Timed() { prof_mark(h, s, cls); }
};

// One decoder stack as the prefill chain sees it, and the buffers the chain works in.
struct Stack {
  const kvp_model_shape* m;
  const ModelW* w;
  const float2* rope;
  bool mfma;              // bf16 MFMA kernels serve this stack
  bool is_base;           // which stack of the handle (for the per-layer widths)
};
struct PrefillBufs {   // byte offsets into the workspace
  size_t x, h, q, attn, gu, act, vt;
  size_t vt_stride = 0;   // > 0: every layer keeps its transposed values (layer l at vt + l * vt_stride), the last included
};

// Causal pass of a stack over B x T_len tokens.  kv_of(l) names where layer l's keys (post-rotary)
// and values go, token-major [B*T][n_kv*hd]; kv_ready(l) is called once they are enqueued.  With
// truncate_last the last layer stops after its key / value projections.
template <typename T, typename KVOf, typename Hook>
int run_stack(kvp_handle* h, const Stack& st, const PrefillBufs& pb, char* ws, const int32_t* tokens, int B, int T_len,
              hipStream_t s, bool truncate_last, KVOf&& kv_of, Hook&& kv_ready) {
  const kvp_config& c = h->cfg;
  const ModelW& mw = *st.w;
  const kvp_model_shape& m_stack = *st.m;
  int N = B * T_len, d = m_stack.d_model, hd = m_stack.head_dim;
  float* x = reinterpret_cast<float*>(ws + pb.x);
  T* hbuf = reinterpret_cast<T*>(ws + pb.h);
  T* q = reinterpret_cast<T*>(ws + pb.q);
  T* attn = reinterpret_cast<T*>(ws + pb.attn);
  T* gu = reinterpret_cast<T*>(ws + pb.gu);
  T* act = reinterpret_cast<T*>(ws + pb.act);
  const bool mf = st.mfma;
  const bool qkn = mw.qk_norm();
  if (qkn && !mw.k_norm[0]) return fail(KVP_ERR_NULL, "k_norm gains of this stack were not given to kvp_load_weights");
  for (int l = 0; l < m_stack.n_layers; ++l) {
    const bool last = truncate_last && (l == m_stack.n_layers - 1);
    const kvp_model_shape m = h->layer_shape(st.is_base, l);     // this layer's widths
    const int qd = m.n_q_heads * hd, Ka = m.n_kv_heads * hd, f = m.ffn_dim;
    T *kl, *vl;
    kv_of(l, kl, vl);
    const T* wq = (const T*)mw.wq[l];
    const T* wk = (const T*)mw.wk[l];
    const T* wv = (const T*)mw.wv[l];
    if (l == 0) {
      Timed t(h, s, KVP_KC_EMBED_NORM);
      launch_embed_rmsnorm<T, T>(tokens, 1, 0, (const T*)mw.embed, c.vocab, (const T*)mw.attn_norm[0], x, hbuf,
                                 N, d, c.rms_eps, h->flags, s);
    } else {
      Timed t(h, s, KVP_KC_EMBED_NORM);
      launch_rmsnorm<T, T>(x, (const T*)mw.attn_norm[l], hbuf, N, d, c.rms_eps, s);
    }
    // Q, K, V projections with rotary on q and k.  A truncated last layer needs K and V only:
    // everything after them feeds the auxiliary logits, which inference never reads (Sec. 4.3
    // "Auxiliary loss").
    if (mf) {
      Timed t(h, s, KVP_KC_AUX_GEMM);
      mfma_qkv_rope((const bf16*)hbuf, last ? nullptr : (const bf16*)wq, (const bf16*)wk, (const bf16*)wv, (bf16*)q,
                    (bf16*)kl, (bf16*)vl, (last && !pb.vt_stride) ? nullptr : (bf16*)(ws + pb.vt + l * pb.vt_stride), N, d,
                    m.n_q_heads, m.n_kv_heads, T_len, st.rope, !qkn, s);
    } else {
      if (!last) {
        Timed t(h, s, KVP_KC_AUX_GEMM);
        launch_gemm_store<T>(hbuf, d, wq, d, q, qd, N, qd, d, s);
      }
      { Timed t(h, s, KVP_KC_AUX_GEMM); launch_gemm_store<T>(hbuf, d, wk, d, kl, Ka, N, Ka, d, s); }
      { Timed t(h, s, KVP_KC_AUX_GEMM); launch_gemm_store<T>(hbuf, d, wv, d, vl, Ka, N, Ka, d, s); }
      if (!qkn) {
        if (!last) { Timed t(h, s, KVP_KC_EMBED_NORM); launch_rope<T>(q, qd, N, m.n_q_heads, hd, T_len, st.rope, s); }
        { Timed t(h, s, KVP_KC_EMBED_NORM); launch_rope<T>(kl, Ka, N, m.n_kv_heads, hd, T_len, st.rope, s); }
      }
    }
    if (qkn) {   // query / key normalisation, then the rotation the projections left out
      if (!last) { Timed t(h, s, KVP_KC_EMBED_NORM);
                   launch_head_norm<T, T>(q, (const T*)mw.q_norm[l], (size_t)N, m.n_q_heads, hd, c.rms_eps, true, T_len, st.rope, s); }
      { Timed t(h, s, KVP_KC_EMBED_NORM);
        launch_head_norm<T, T>(kl, (const T*)mw.k_norm[l], (size_t)N, m.n_kv_heads, hd, c.rms_eps, true, T_len, st.rope, s); }
    }
    kv_ready(l);          // K[l], V[l] are enqueued: whatever consumes them may go
    if (last) break;
    if (mf) {
      Timed t(h, s, KVP_KC_AUX_ATTN);
      mfma_flash_prefill((const bf16*)q, (const bf16*)kl, (const bf16*)(ws + pb.vt + l * pb.vt_stride), (bf16*)attn, B, T_len, m.n_q_heads,
                         m.n_kv_heads, s);
    } else {
      Timed t(h, s, KVP_KC_AUX_ATTN);
      launch_attn_prefill_generic<T>(q, kl, vl, attn, B, T_len, m.n_q_heads, m.n_kv_heads, hd, s);
    }
    if (mf) {
      { Timed t(h, s, KVP_KC_AUX_GEMM); mfma_gemm_residual((const bf16*)attn, (const bf16*)mw.wo[l], x, N, d, qd, s); }
      { Timed t(h, s, KVP_KC_EMBED_NORM); launch_rmsnorm<T, T>(x, (const T*)mw.ffn_norm[l], hbuf, N, d, c.rms_eps, s); }
      { Timed t(h, s, KVP_KC_AUX_GEMM);
        mfma_gemm_swiglu((const bf16*)hbuf, (const bf16*)mw.w_gate[l], (const bf16*)mw.w_up[l], (bf16*)act, N, f, d, s); }
      { Timed t(h, s, KVP_KC_AUX_GEMM); mfma_gemm_residual((const bf16*)act, (const bf16*)mw.w_down[l], x, N, d, f, s); }
    } else {
      { Timed t(h, s, KVP_KC_AUX_GEMM); launch_gemm_residual<T>(attn, qd, (const T*)mw.wo[l], qd, x, d, N, d, qd, s); }
      { Timed t(h, s, KVP_KC_EMBED_NORM); launch_rmsnorm<T, T>(x, (const T*)mw.ffn_norm[l], hbuf, N, d, c.rms_eps, s); }
      { Timed t(h, s, KVP_KC_AUX_GEMM); launch_gemm_store<T>(hbuf, d, (const T*)mw.w_gate[l], d, gu, 2 * f, N, f, d, s); }
      { Timed t(h, s, KVP_KC_AUX_GEMM); launch_gemm_store<T>(hbuf, d, (const T*)mw.w_up[l], d, gu + f, 2 * f, N, f, d, s); }
      { Timed t(h, s, KVP_KC_EMBED_NORM); launch_silu_mul<T>(gu, act, (size_t)N, f, s); }
      { Timed t(h, s, KVP_KC_AUX_GEMM); launch_gemm_residual<T>(act, f, (const T*)mw.w_down[l], f, x, d, N, d, f, s); }
    }
  }
  return KVP_OK;
}

// a, KV_A <- A(I)  (Sec. 4.1): the auxiliary stack, keys / values of every layer kept in the workspace
template <typename T, typename Hook>
int run_aux(kvp_handle* h, const Workspace& w, char* ws, const int32_t* tokens, int B, int T_len, hipStream_t s,
            Hook&& kv_ready) {
  const kvp_model_shape& m = h->cfg.aux;
  const size_t per_layer = (size_t)B * T_len * m.n_kv_heads * m.head_dim;
  T* aux_k = reinterpret_cast<T*>(ws + w.aux_k);
  T* aux_v = reinterpret_cast<T*>(ws + w.aux_v);
  Stack st{&h->cfg.aux, &h->aux, h->rope_aux, h->use_mfma, false};
  PrefillBufs pb{w.x, w.h, w.q, w.attn, w.gu, w.act, w.vt, w.vt_layer};
  return run_stack<T>(h, st, pb, ws, tokens, B, T_len, s, true,
                      [&](int l, T*& kl, T*& vl) { kl = aux_k + l * per_layer; vl = aux_v + l * per_layer; }, kv_ready);
}

// K^_i = K_A[j_i] W_K,i^T and V^_i = V_A[j_i] W_V,i^T, written straight into the caller's cache
// [L_B][B][n_kv_b][T_cap][hd]  (Sec. 4.2 "Predictor Networks").
template <typename T>
int run_predict(kvp_handle* h, const Workspace& w, char* ws, int B, int T_len, void* k_cache, void* v_cache,
                int64_t T_cap, hipStream_t s, int i0 = 0, int i1 = -1) {
  const kvp_config& c = h->cfg;
  int N = B * T_len;
  const int hd_a = c.aux.head_dim, hd_b = c.base.head_dim;
  const T* aux_k = reinterpret_cast<const T*>(ws + w.aux_k);
  const T* aux_v = reinterpret_cast<const T*>(ws + w.aux_v);
  // blocks of the widest layer's size; a narrower layer's dense array sits at the start of its block
  const size_t aux_block = (size_t)N * c.aux.n_kv_heads * hd_a;
  const size_t layer_elems = (size_t)B * c.base.n_kv_heads * T_cap * hd_b;
  if (i1 < 0) i1 = c.base.n_layers;
  if (h->use_mfma) {
    // one batched launch per run of base layers of one width whose auxiliary layers have one width
    // (the kernel finds each problem's auxiliary layer through the layer map)
    for (int i = i0; i < i1;) {
      int e = i + 1;
      while (e < i1 && h->a_nkv[h->layer_map[e]] == h->a_nkv[h->layer_map[i]] && h->b_nkv[e] == h->b_nkv[i]) ++e;
      const int Ka = h->a_nkv[h->layer_map[i]] * hd_a, Kb = h->b_nkv[i] * hd_b;
      Timed t(h, s, KVP_KC_PREDICTOR);
      int rc = mfma_predictor(h, h->mfma_tables, (const bf16*)aux_k, (const bf16*)aux_v, (bf16*)k_cache, (bf16*)v_cache, B,
                              T_len, T_cap, i, e, Ka, Kb, h->b_nkv[i], aux_block, layer_elems, s);
      if (rc != KVP_OK) return rc;
      i = e;
    }
    return KVP_OK;
  }
  for (int i = i0; i < i1; ++i) {
    int j = h->layer_map[i];
    const int Ka = h->a_nkv[j] * hd_a, Kb = h->b_nkv[i] * hd_b;
    const T* ka = aux_k + (size_t)j * aux_block;
    const T* va = aux_v + (size_t)j * aux_block;
    { Timed t(h, s, KVP_KC_PREDICTOR);
      launch_gemm_cache<T>(ka, Ka, (const T*)h->pred_wk[i], Ka, (T*)k_cache + i * layer_elems, T_len, T_cap,
                           h->b_nkv[i], hd_b, N, Kb, Ka, s); }
    { Timed t(h, s, KVP_KC_PREDICTOR);
      launch_gemm_cache<T>(va, Ka, (const T*)h->pred_wv[i], Ka, (T*)v_cache + i * layer_elems, T_len, T_cap,
                           h->b_nkv[i], hd_b, N, Kb, Ka, s); }
  }
  return KVP_OK;
}

// Attention of base layer i with the predictor absorbed (Sec. 4.2 "Predictor Networks": the maps are
// linear): q [B][n_q][hd] unrotated -> attention output [B][n_q*hd], read from the AUXILIARY cache of
// layer j_i in the workspace instead of the predicted cache.  See kernels_absorbed.hip.
template <typename T>
int absorbed_attention(kvp_handle* h, const Workspace& w, char* ws, int i, int B, int T_len, const float* bq, float* out,
                       bf16* out_hi, bf16* out_lo, hipStream_t s) {
  const kvp_config& c = h->cfg;
  const int j = h->layer_map[i], hd = c.base.head_dim, n_q = h->b_nq[i], n_kv = h->b_nkv[i];
  const int Ka = h->a_nkv[j] * c.aux.head_dim;
  if (!absorbed_attn_supported(Ka) || n_q / n_kv > 8 || hd > 256)
    return fail(KVP_ERR_UNIMPLEMENTED, "absorbed base step: auxiliary width %d (a power of two in 16..512), query group %d (<= 8), "
                "head_dim %d (<= 256) not served", Ka, n_q / n_kv, hd);
  const size_t aux_block = (size_t)B * T_len * c.aux.n_kv_heads * c.aux.head_dim;     // block of the widest layer
  const T* ka = reinterpret_cast<const T*>(ws + w.aux_k) + (size_t)j * aux_block;
  const T* va = reinterpret_cast<const T*>(ws + w.aux_v) + (size_t)j * aux_block;
  float* qw = reinterpret_cast<float*>(ws + w.qw);
  float* rw = reinterpret_cast<float*>(ws + w.rw);
  float* part = reinterpret_cast<float*>(ws + w.part);
  bool ok;
  { Timed t(h, s, KVP_KC_DECODE_ATTN);
    ok = launch_absorb_q<T>(bq, (const T*)h->pred_wk[i], qw, B, n_q, n_kv, hd, Ka, T_len - 1, h->rope_base, s); }
  if (ok) {
    Timed t(h, s, KVP_KC_DECODE_ATTN);
    if (absorbed_on_mfma(h, Ka))
      ok = launch_absorbed_attn_mfma(qw, (const bf16*)ka, (const bf16*)(ws + w.vt + (size_t)j * w.vt_layer), part, rw, B, T_len,
                                     (T_len + 63) / 64 * 64, n_q, Ka, s);
    else
      ok = launch_absorbed_attn<T>(qw, ka, va, part, rw, B, T_len, n_q, Ka, absorbed_splits(h, B, n_q, Ka, w.plan_T), s);
  }
  if (ok) {
    Timed t(h, s, KVP_KC_DECODE_ATTN);
    ok = launch_absorb_o<T>(rw, (const T*)h->pred_wv[i], out, out_hi, out_lo, B, n_q, n_kv, hd, Ka, s);
  }
  if (!ok) return fail(KVP_ERR_UNIMPLEMENTED, "absorbed base step: a kernel refused layer %d", i);
  return KVP_OK;
}

// bf16 base step on the matrix cores: activations are handed from kernel to kernel as bf16
// high / low halves, RMSNorm is folded into the producers / consumers (see kernels_base_chain.hip).
struct BaseChain {
  kvp_handle* h; const Workspace& w; char* ws; const int32_t* tokens; int B, T_len;
  const void* k_cache; const void* v_cache; int64_t T_cap; float* logits; int32_t* argmax; hipStream_t s;
  // Generation step (append >= 0): `tokens` holds one token per sequence, its key / value are
  // computed, rotated to position `append` and stored in that cache slot, and attention reads
  // append + 1 entries.  First-token step (append < 0): T_len prompt tokens, T_len predicted entries.
  int append = -1;
  bool absorbed = false;   // first-token step reading the auxiliary cache through the predictor's maps (no k_cache / v_cache)
  int parts = 1;   // the embedding kernel emits one sum of squares per sequence

  float* f32(size_t off) const { return reinterpret_cast<float*>(ws + off); }
  bf16* b16(size_t off) const { return reinterpret_cast<bf16*>(ws + off); }

  void begin() {
    const kvp_config& c = h->cfg;
    Timed t(h, s, KVP_KC_EMBED_NORM);
    launch_base_embed(tokens, append >= 0 ? 1 : T_len, (const bf16*)h->base.embed, c.vocab,
                      (const bf16*)h->base.attn_norm[0], f32(w.y), b16(w.uh), b16(w.ul), f32(w.ssq), B, c.base.d_model,
                      h->flags, s);
  }
  int layer(int i) {
    const kvp_config& c = h->cfg;
    const kvp_model_shape m = h->layer_shape(true, i);            // this layer's widths
    const int d = m.d_model, hd = m.head_dim, qd = m.n_q_heads * hd, f = m.ffn_dim;
    const size_t layer_elems = (size_t)B * c.base.n_kv_heads * T_cap * hd;   // block of the widest layer
    const int n_splits = decode_attn_splits(B, m.n_kv_heads, w.plan_T);
    bf16 *uh = b16(w.uh), *ul = b16(w.ul), *oh = b16(w.oh), *ol = b16(w.ol), *ah = b16(w.ah), *al = b16(w.al);
    float *y = f32(w.y), *bq = f32(w.bq), *ssq = f32(w.ssq);
    { Timed t(h, s, KVP_KC_BASE_GEMV);
      launch_chain_project((const bf16*)h->base.wq[i], uh, ul, ssq, parts, c.rms_eps, bq, B, qd, d, s); }
    if (h->base.qk_norm()) { Timed t(h, s, KVP_KC_EMBED_NORM);
      launch_head_norm<float, bf16>(bq, (const bf16*)h->base.q_norm[i], (size_t)B, m.n_q_heads, hd, c.rms_eps, false, 1, nullptr, s); }
    const int attn_len = append >= 0 ? append + 1 : T_len;
    if (append >= 0) {
      const int kd = m.n_kv_heads * hd;
      { Timed t(h, s, KVP_KC_BASE_GEMV);
        launch_chain_project((const bf16*)h->base.wk[i], uh, ul, ssq, parts, c.rms_eps, f32(w.bk), B, kd, d, s); }
      { Timed t(h, s, KVP_KC_BASE_GEMV);
        launch_chain_project((const bf16*)h->base.wv[i], uh, ul, ssq, parts, c.rms_eps, f32(w.bv), B, kd, d, s); }
      if (h->base.qk_norm()) { Timed t(h, s, KVP_KC_EMBED_NORM);
        launch_head_norm<float, bf16>(f32(w.bk), (const bf16*)h->base.k_norm[i], (size_t)B, m.n_kv_heads, hd, c.rms_eps, false, 1, nullptr, s); }
      { Timed t(h, s, KVP_KC_EMBED_NORM);
        launch_kv_append<bf16>(f32(w.bk), f32(w.bv), (bf16*)const_cast<void*>(k_cache) + i * layer_elems,
                               (bf16*)const_cast<void*>(v_cache) + i * layer_elems, B, append, T_cap, m.n_kv_heads, hd,
                               h->rope_base, s); }
    }
    // One or two sequences: the output projection merges the attention splits in its prologue.  (With more
    // sequences every block of the projection would pull all partials -- n_splits x B x n_q x hd floats, 0.5 MB at
    // 4 x 8192 tokens of the 8B-class shapes -- through its CU's L1; measured 18 us slower per layer than the
    // 4 us combine launch it saves.)
    const bool merge_in_o = !absorbed && B <= 2 && n_splits <= 8 && hd % 8 == 0;
    if (absorbed) {
      int rc = absorbed_attention<bf16>(h, w, ws, i, B, T_len, bq, nullptr, oh, ol, s);
      if (rc != KVP_OK) return rc;
    } else { Timed t(h, s, KVP_KC_DECODE_ATTN);
      if (!launch_decode_attn<bf16>(bq, (const bf16*)k_cache + i * layer_elems, (const bf16*)v_cache + i * layer_elems,
                                    f32(w.part), nullptr, merge_in_o ? nullptr : oh, merge_in_o ? nullptr : ol, B, attn_len,
                                    T_cap, m.n_q_heads, m.n_kv_heads, hd, n_splits, h->rope_base, s))
        return fail(KVP_ERR_BAD_CONFIG, "decode attention: unsupported head_dim %d / group %d", hd, m.n_q_heads / m.n_kv_heads); }
    { Timed t(h, s, KVP_KC_BASE_GEMV);
      if (!merge_in_o ||
          !launch_chain_residual_merge((const bf16*)h->base.wo[i], f32(w.part), n_splits, m.n_q_heads, hd, y,
                                       (const bf16*)h->base.ffn_norm[i], uh, ul, ssq, B, d, qd, s)) {
        if (merge_in_o) return fail(KVP_ERR_BAD_CONFIG, "merging output projection refused head_dim %d x %d heads", hd, m.n_q_heads);
        launch_chain_residual((const bf16*)h->base.wo[i], oh, ol, y, (const bf16*)h->base.ffn_norm[i], uh, ul, ssq, B, d, qd, s);
      } }
    parts = chain_ssq_parts(d, B);
    { Timed t(h, s, KVP_KC_BASE_GEMV);
      launch_chain_swiglu((const bf16*)h->base.w_gate[i], (const bf16*)h->base.w_up[i], uh, ul, ssq, parts, c.rms_eps, ah, al,
                          B, f, d, s); }
    const void* gain_next = (i + 1 < m.n_layers) ? h->base.attn_norm[i + 1] : h->base.final_norm;
    { Timed t(h, s, KVP_KC_BASE_GEMV);
      launch_chain_residual((const bf16*)h->base.w_down[i], ah, al, y, (const bf16*)gain_next, uh, ul, ssq, B, d, f, s); }
    return KVP_OK;
  }
  void end() {
    const kvp_config& c = h->cfg;
    float* lg = logits ? logits : f32(w.logits);
    { Timed t(h, s, KVP_KC_BASE_GEMV);
      launch_chain_project((const bf16*)h->base.lm_head, b16(w.uh), b16(w.ul), f32(w.ssq), parts, c.rms_eps, lg, B, c.vocab,
                           c.base.d_model, s); }
    if (argmax) {
      Timed t(h, s, KVP_KC_ARGMAX);
      launch_argmax(lg, argmax, B, c.vocab, s);
    }
  }
};

int run_base_bf16(kvp_handle* h, const Workspace& w, char* ws, const int32_t* tokens, int B, int T_len,
                  const void* k_cache, const void* v_cache, int64_t T_cap, float* logits, int32_t* argmax, hipStream_t s,
                  int append = -1, bool absorbed = false) {
  BaseChain bc{h, w, ws, tokens, B, T_len, k_cache, v_cache, T_cap, logits, argmax, s};
  bc.append = append;
  bc.absorbed = absorbed;
  bc.begin();
  for (int i = 0; i < h->cfg.base.n_layers; ++i) {
    int rc = bc.layer(i);
    if (rc != KVP_OK) return rc;
  }
  bc.end();
  return KVP_OK;
}

// The auxiliary chain and the base chain are each a sequence of dependent kernels; at small
// B x T neither fills 256 CUs, and base layer i needs only the auxiliary layers up to j_i.  So the
// whole path is issued on two streams: the caller's stream runs the auxiliary prefill and records
// an event when a layer's K/V are done; an internal stream waits for it, runs the predictor for
// the base layers that layer feeds (for short prompts the caller's stream runs it, before the event),
// then every base layer that is now unblocked.  The caller's
// stream finally waits for the internal one, so from outside the call is still "enqueued on the
// caller's stream".  At large B x T the gain is what of the base step fits beside the prefill.
// With the predictor absorbed into the base step (absorbed), the base chain waits for the auxiliary
// layer itself, and the predicted cache (predict) is written by the caller's stream after the
// auxiliary prefill, beside the last base layers: the first token no longer waits for it.
int run_overlapped(kvp_handle* h, const Workspace& w, char* ws, const int32_t* tokens, int B, int T_len, void* k_cache,
                   void* v_cache, int64_t T_cap, float* logits, int32_t* argmax, hipStream_t s, bool absorbed = false,
                   bool predict = true) {
  const kvp_config& c = h->cfg;
  const int LB = c.base.n_layers;
  hipStream_t sb = h->side;
  if (hipEventRecord(h->ev_start, s) != hipSuccess || hipStreamWaitEvent(sb, h->ev_start, 0) != hipSuccess)
    return fail(KVP_ERR_HIP, "could not fork the internal stream");
  BaseChain bc{h, w, ws, tokens, B, T_len, k_cache, v_cache, T_cap, logits, argmax, sb};
  bc.absorbed = absorbed;
  bc.begin();
  int next_base = 0, rc_hook = KVP_OK;
  // Which stream runs the predictor.  Up to some ten thousand tokens its launches are short and the internal stream's
  // chain of base-step launches is the critical path, so the predictor goes onto the caller's stream, between the
  // auxiliary layers (measured: TTFT -2.5 % at 1 x 1024 tokens, -1.7 % at 4 x 2048, -2 % at 8 x 2048); at 32768 tokens
  // it stays on the internal stream, where its cache writes run beside the auxiliary GEMMs (there the other order is
  // 0.2 % slower).
  const bool pred_main = h->pred_main >= 0 ? h->pred_main == 1 : (size_t)B * T_len <= 16384;   // (KVP_PRED_MAIN=0|1 at load time overrides)
  auto predict_layer = [&](int l, hipStream_t st) {   // predictor for every run of base layers fed by auxiliary layer l
    for (int i = 0; i < LB && !absorbed;) {
      if (h->layer_map[i] != l) { ++i; continue; }
      int i1 = i;
      while (i1 < LB && h->layer_map[i1] == l) ++i1;
      int rc = run_predict<bf16>(h, w, ws, B, T_len, k_cache, v_cache, T_cap, st, i, i1);
      if (rc != KVP_OK) { rc_hook = rc; return; }
      i = i1;
    }
  };
  auto kv_ready = [&](int l) {
    if (rc_hook != KVP_OK) return;
    if (pred_main) predict_layer(l, s);
    if (rc_hook != KVP_OK) return;
    if (hipEventRecord(h->ev_kv[l], s) != hipSuccess || hipStreamWaitEvent(sb, h->ev_kv[l], 0) != hipSuccess) {
      rc_hook = fail(KVP_ERR_HIP, "could not link the streams at auxiliary layer %d", l);
      return;
    }
    if (!pred_main) predict_layer(l, sb);
    if (rc_hook != KVP_OK) return;
    // base layers run in order: layer i may go once every auxiliary layer up to j_i is enqueued
    while (next_base < LB && h->layer_map[next_base] <= l) {
      int rc = bc.layer(next_base);
      if (rc != KVP_OK) { rc_hook = rc; return; }
      ++next_base;
    }
  };
  int rc = run_aux<bf16>(h, w, ws, tokens, B, T_len, s, kv_ready);
  if (rc == KVP_OK) rc = rc_hook;
  if (rc == KVP_OK && absorbed && predict) rc = run_predict<bf16>(h, w, ws, B, T_len, k_cache, v_cache, T_cap, s);
  for (; rc == KVP_OK && next_base < LB; ++next_base) rc = bc.layer(next_base);
  if (rc == KVP_OK) bc.end();
  // The internal stream joins the caller's stream on the error paths too: whatever was enqueued on it
  // before the failure must not outlive the call (and a capture through the caller's stream stays valid).
  if (hipEventRecord(h->ev_done, sb) != hipSuccess || hipStreamWaitEvent(s, h->ev_done, 0) != hipSuccess)
    return rc != KVP_OK ? rc : fail(KVP_ERR_HIP, "could not join the internal stream");
  return rc;
}

// b <- B(I[-1], KV^_B): the base model computes a query only; keys and values come from the
// predicted cache (Sec. 4.1 "Inference").
template <typename T>
int run_base(kvp_handle* h, const Workspace& w, char* ws, const int32_t* tokens, int B, int T_len, const void* k_cache,
             const void* v_cache, int64_t T_cap, float* logits, int32_t* argmax, hipStream_t s, int append = -1,
             bool absorbed = false) {
  const kvp_config& c = h->cfg;
  const int d = c.base.d_model, hd = c.base.head_dim, n_layers = c.base.n_layers;
  float* y = reinterpret_cast<float*>(ws + w.y);
  float* bq = reinterpret_cast<float*>(ws + w.bq);
  float* battn = reinterpret_cast<float*>(ws + w.battn);
  float* bact = reinterpret_cast<float*>(ws + w.bact);
  float* part = reinterpret_cast<float*>(ws + w.part);
  float* lg = logits ? logits : reinterpret_cast<float*>(ws + w.logits);
  size_t layer_elems = (size_t)B * c.base.n_kv_heads * T_cap * hd;      // block of the widest layer
  {
    Timed t(h, s, KVP_KC_EMBED_NORM);
    // generation step (append >= 0): one token per sequence; else the last of T_len prompt tokens
    launch_embed_rmsnorm<T, float>(tokens, append >= 0 ? 1 : T_len, append >= 0 ? 0 : T_len - 1, (const T*)h->base.embed,
                                   c.vocab, nullptr, y, nullptr, B, d, c.rms_eps, h->flags, s);
  }
  const int attn_len = append >= 0 ? append + 1 : T_len;
  for (int i = 0; i < n_layers; ++i) {
    const kvp_model_shape m = h->layer_shape(true, i);              // this layer's widths
    const int qd = m.n_q_heads * hd, f = m.ffn_dim;
    const int n_splits = decode_attn_splits(B, m.n_kv_heads, w.plan_T);
    { Timed t(h, s, KVP_KC_BASE_GEMV);
      launch_gemv<T>(0, true, (const T*)h->base.wq[i], nullptr, y, (const T*)h->base.attn_norm[i], bq, B, qd, d, c.rms_eps, s); }
    if (h->base.qk_norm()) { Timed t(h, s, KVP_KC_EMBED_NORM);
      launch_head_norm<float, T>(bq, (const T*)h->base.q_norm[i], (size_t)B, m.n_q_heads, hd, c.rms_eps, false, 1, nullptr, s); }
    if (append >= 0) {   // own key / value of the new token into cache slot `append`
      const int kd = m.n_kv_heads * hd;
      float* bk = reinterpret_cast<float*>(ws + w.bk);
      float* bv = reinterpret_cast<float*>(ws + w.bv);
      { Timed t(h, s, KVP_KC_BASE_GEMV);
        launch_gemv<T>(0, true, (const T*)h->base.wk[i], nullptr, y, (const T*)h->base.attn_norm[i], bk, B, kd, d, c.rms_eps, s); }
      { Timed t(h, s, KVP_KC_BASE_GEMV);
        launch_gemv<T>(0, true, (const T*)h->base.wv[i], nullptr, y, (const T*)h->base.attn_norm[i], bv, B, kd, d, c.rms_eps, s); }
      if (h->base.qk_norm()) { Timed t(h, s, KVP_KC_EMBED_NORM);
        launch_head_norm<float, T>(bk, (const T*)h->base.k_norm[i], (size_t)B, m.n_kv_heads, hd, c.rms_eps, false, 1, nullptr, s); }
      { Timed t(h, s, KVP_KC_EMBED_NORM);
        launch_kv_append<T>(bk, bv, (T*)const_cast<void*>(k_cache) + i * layer_elems, (T*)const_cast<void*>(v_cache) + i * layer_elems,
                            B, append, T_cap, m.n_kv_heads, hd, h->rope_base, s); }
    }
    if (absorbed) {
      int rc = absorbed_attention<T>(h, w, ws, i, B, T_len, bq, battn, nullptr, nullptr, s);
      if (rc != KVP_OK) return rc;
    } else { Timed t(h, s, KVP_KC_DECODE_ATTN);
      if (!launch_decode_attn<T>(bq, (const T*)k_cache + i * layer_elems, (const T*)v_cache + i * layer_elems, part, battn,
                                 nullptr, nullptr, B, attn_len, T_cap, m.n_q_heads, m.n_kv_heads, hd, n_splits, h->rope_base, s))
        return fail(KVP_ERR_BAD_CONFIG, "decode attention: unsupported head_dim %d / group %d", hd, m.n_q_heads / m.n_kv_heads); }
    { Timed t(h, s, KVP_KC_BASE_GEMV);
      launch_gemv<T>(1, false, (const T*)h->base.wo[i], nullptr, battn, nullptr, y, B, d, qd, c.rms_eps, s); }
    { Timed t(h, s, KVP_KC_BASE_GEMV);
      launch_gemv<T>(2, true, (const T*)h->base.w_gate[i], (const T*)h->base.w_up[i], y, (const T*)h->base.ffn_norm[i], bact,
                     B, f, d, c.rms_eps, s); }
    { Timed t(h, s, KVP_KC_BASE_GEMV);
      launch_gemv<T>(1, false, (const T*)h->base.w_down[i], nullptr, bact, nullptr, y, B, d, f, c.rms_eps, s); }
  }
  { Timed t(h, s, KVP_KC_BASE_GEMV);
    launch_gemv<T>(0, true, (const T*)h->base.lm_head, nullptr, y, (const T*)h->base.final_norm, lg, B, c.vocab, d, c.rms_eps, s); }
  if (argmax) {
    Timed t(h, s, KVP_KC_ARGMAX);
    launch_argmax(lg, argmax, B, c.vocab, s);
  }
  return KVP_OK;
}

template <typename T>
int run_stages(kvp_handle* h, uint32_t stages, const Workspace& w, char* ws, const int32_t* tokens, int B, int T_len,
               void* k_cache, void* v_cache, int64_t T_cap, float* logits, int32_t* argmax, hipStream_t s) {
  int rc = KVP_OK;
  const bool absorbed = (stages & KVP_STAGE_BASE_ABSORBED) != 0;
  const bool whole = stages == KVP_STAGE_ALL || stages == (KVP_STAGE_AUX | KVP_STAGE_BASE_ABSORBED) ||
                     stages == (KVP_STAGE_AUX | KVP_STAGE_PREDICT | KVP_STAGE_BASE_ABSORBED);
  if (whole && h->overlap && !h->prof_on && sizeof(T) == 2) {
    rc = run_overlapped(h, w, ws, tokens, B, T_len, k_cache, v_cache, T_cap, logits, argmax, s, absorbed,
                        (stages & KVP_STAGE_PREDICT) != 0);
    if (rc != KVP_OK) return rc;
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(KVP_ERR_HIP, "HIP error after launch: %s", hipGetErrorString(e));
    return KVP_OK;
  }
  prof_mark(h, s, -1);
  if (stages & KVP_STAGE_AUX) rc = run_aux<T>(h, w, ws, tokens, B, T_len, s, [](int) {});
  if (rc == KVP_OK && (stages & KVP_STAGE_PREDICT)) rc = run_predict<T>(h, w, ws, B, T_len, k_cache, v_cache, T_cap, s);
  if (rc == KVP_OK && (stages & (KVP_STAGE_BASE | KVP_STAGE_BASE_ABSORBED))) {
    if (h->cfg.dtype == KVP_DTYPE_BF16 && !h->force_generic)
      rc = run_base_bf16(h, w, ws, tokens, B, T_len, k_cache, v_cache, T_cap, logits, argmax, s, -1, absorbed);
    else
      rc = run_base<T>(h, w, ws, tokens, B, T_len, k_cache, v_cache, T_cap, logits, argmax, s, -1, absorbed);
  }
  if (rc != KVP_OK) return rc;
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(KVP_ERR_HIP, "HIP error after launch: %s", hipGetErrorString(e));
  return KVP_OK;
}

// ---------------------------------------------------------------------------------------
// Ordinary inference of one model alone (Sec. 6.3 "Timing Experiments": the time to first
// token of the base model and of the small model, against which KV Prediction is measured): the
// same prefill chain on that model's stack, every layer complete, then final norm + LM head on
// the last prompt position.
// ---------------------------------------------------------------------------------------
struct RefWorkspace {
  PrefillBufs pb;
  size_t kl, vl, y, logits, total;
};
bool stack_mfma(const kvp_handle* h, const kvp_model_shape& m) {
  if (h->cfg.dtype != KVP_DTYPE_BF16 || h->force_generic) return false;
  const bool is_base = &m == &h->cfg.base;
  for (int l = 0; l < m.n_layers; ++l) {         // every layer's widths must suit the MFMA kernels
    const kvp_model_shape ml = h->layer_shape(is_base, l);
    if (!mfma_shape_supported(&ml)) return false;
  }
  return true;
}
RefWorkspace plan_reference(const kvp_handle* h, const kvp_model_shape& m, int B, int T) {
  size_t N = (size_t)B * T, es = h->esize;
  size_t qd = (size_t)m.n_q_heads * m.head_dim, kd = (size_t)m.n_kv_heads * m.head_dim;
  const bool mf = stack_mfma(h, m);
  RefWorkspace r{};
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
  r.pb.x = take(N * m.d_model * sizeof(float));
  r.pb.h = take(N * m.d_model * es);
  r.pb.q = take(N * qd * es);
  r.pb.attn = take(N * qd * es);
  r.pb.gu = take(mf ? 0 : N * 2 * (size_t)m.ffn_dim * es);
  r.pb.act = take(N * (size_t)m.ffn_dim * es);
  r.pb.vt = take(mf ? mfma_vt_bytes_shape(&m, B, T) : 0);
  r.kl = take(N * kd * es);
  r.vl = take(N * kd * es);
  r.y = take((size_t)B * m.d_model * sizeof(float));
  r.logits = take((size_t)B * h->cfg.vocab * sizeof(float));
  r.total = off;
  return r;
}
template <typename T>
int run_reference(kvp_handle* h, const kvp_model_shape& m, const ModelW& mw, const float2* rope, const RefWorkspace& r,
                  char* ws, const int32_t* tokens, int B, int T_len, void* k_cache, void* v_cache, int64_t T_cap,
                  float* logits, int32_t* argmax, hipStream_t s) {
  const kvp_config& c = h->cfg;
  T* kl0 = reinterpret_cast<T*>(ws + r.kl);
  T* vl0 = reinterpret_cast<T*>(ws + r.vl);
  const size_t layer_elems = (size_t)B * m.n_kv_heads * T_cap * m.head_dim;   // block of the widest layer
  const bool is_base = &m == &h->cfg.base;
  Stack st{&m, &mw, rope, stack_mfma(h, m), is_base};
  prof_mark(h, s, -1);
  int rc = run_stack<T>(h, st, r.pb, ws, tokens, B, T_len, s, false,
                        [&](int, T*& kl, T*& vl) { kl = kl0; vl = vl0; },
                        [&](int l) {
                          if (!k_cache) return;       // the caller keeps the model's own cache, in cache layout
                          Timed t(h, s, KVP_KC_EMBED_NORM);
                          const int n_kv = h->layer_shape(is_base, l).n_kv_heads;
                          launch_rows_to_cache<T>(kl0, (T*)k_cache + l * layer_elems, B, T_len, T_cap, n_kv, m.head_dim, s);
                          launch_rows_to_cache<T>(vl0, (T*)v_cache + l * layer_elems, B, T_len, T_cap, n_kv, m.head_dim, s);
                        });
  if (rc != KVP_OK) return rc;
  float* y = reinterpret_cast<float*>(ws + r.y);
  float* lg = logits ? logits : reinterpret_cast<float*>(ws + r.logits);
  { Timed t(h, s, KVP_KC_EMBED_NORM);
    launch_gather_last_rows(reinterpret_cast<const float*>(ws + r.pb.x), y, B, T_len, m.d_model, s); }
  { Timed t(h, s, KVP_KC_BASE_GEMV);
    launch_gemv<T>(0, true, (const T*)mw.lm_head, nullptr, y, (const T*)mw.final_norm, lg, B, c.vocab, m.d_model, c.rms_eps, s); }
  if (argmax) {
    Timed t(h, s, KVP_KC_ARGMAX);
    launch_argmax(lg, argmax, B, c.vocab, s);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(KVP_ERR_HIP, "HIP error after launch: %s", hipGetErrorString(e));
  return KVP_OK;
}

int check_shape(const char* name, const kvp_model_shape& m) {
  if (m.n_layers < 1 || m.d_model < 8 || m.n_q_heads < 1 || m.n_kv_heads < 1 || m.head_dim < 8 || m.ffn_dim < 8)
    return fail(KVP_ERR_BAD_CONFIG, "%s: non-positive or too small dimension", name);
  if (!m.layer_n_q_heads && m.n_q_heads % m.n_kv_heads)      // (per-layer widths are checked layer by layer)
    return fail(KVP_ERR_BAD_CONFIG, "%s: n_q_heads %% n_kv_heads != 0", name);
  if (m.d_model % 8 || m.ffn_dim % 8 || m.head_dim % 8)
    return fail(KVP_ERR_BAD_CONFIG, "%s: d_model, ffn_dim and head_dim must be multiples of 8", name);
  if (m.head_dim > 256) return fail(KVP_ERR_BAD_CONFIG, "%s: head_dim > 256", name);
  return KVP_OK;
}

// Per-layer widths of a stack: copies of the optional arrays (validated against the scalar
// maxima), or the scalar widths for every layer.
int copy_widths(const char* name, const kvp_model_shape& m, bool is_base, std::vector<int32_t>& nq, std::vector<int32_t>& nkv,
                std::vector<int32_t>& f) {
  const bool any = m.layer_n_q_heads || m.layer_n_kv_heads || m.layer_ffn_dim;
  if (any && !(m.layer_n_q_heads && m.layer_n_kv_heads && m.layer_ffn_dim))
    return fail(KVP_ERR_NULL, "%s: give layer_n_q_heads, layer_n_kv_heads and layer_ffn_dim together or not at all", name);
  nq.assign(m.n_layers, m.n_q_heads); nkv.assign(m.n_layers, m.n_kv_heads); f.assign(m.n_layers, m.ffn_dim);
  if (!any) return KVP_OK;
  int mq = 0, mkv = 0, mf = 0;
  for (int l = 0; l < m.n_layers; ++l) {
    nq[l] = m.layer_n_q_heads[l]; nkv[l] = m.layer_n_kv_heads[l]; f[l] = m.layer_ffn_dim[l];
    if (nq[l] < 1 || nkv[l] < 1 || nq[l] % nkv[l] || f[l] < 8 || f[l] % 8)
      return fail(KVP_ERR_BAD_CONFIG, "%s layer %d: bad widths (%d query heads, %d kv heads, ffn %d)", name, l, nq[l], nkv[l], f[l]);
    if (is_base && !decode_attn_supported(m.head_dim, nq[l] / nkv[l]))
      return fail(KVP_ERR_BAD_CONFIG, "%s layer %d: n_q/n_kv must be one of 1,2,3,4,6,8", name, l);
    mq = nq[l] > mq ? nq[l] : mq; mkv = nkv[l] > mkv ? nkv[l] : mkv; mf = f[l] > mf ? f[l] : mf;
  }
  if (mq != m.n_q_heads || mkv != m.n_kv_heads || mf != m.ffn_dim)
    return fail(KVP_ERR_BAD_CONFIG, "%s: n_q_heads / n_kv_heads / ffn_dim must be the maxima of the per-layer widths", name);
  return KVP_OK;
}

// Every kernel reads weights, caches and logits in 16-byte pieces: rows are multiples of 16 bytes by the shape
// checks, the base addresses are checked here.
bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

int copy_model(const char* name, const kvp_model_shape& m, const kvp_model_weights& src, ModelW& dst, bool is_base) {
  if (!src.embed) return fail(KVP_ERR_NULL, "%s.embed is NULL", name);
  if (!aligned16(src.embed) || !aligned16(src.final_norm) || !aligned16(src.lm_head))
    return fail(KVP_ERR_BAD_CONFIG, "%s.embed / final_norm / lm_head is not 16-byte aligned", name);
  if (is_base && (!src.final_norm || !src.lm_head)) return fail(KVP_ERR_NULL, "%s.final_norm / lm_head is NULL", name);
  dst.embed = src.embed; dst.final_norm = src.final_norm; dst.lm_head = src.lm_head;
  struct { const void* const* p; std::vector<const void*>* v; const char* n; bool optional; } f[] = {
      {src.attn_norm, &dst.attn_norm, "attn_norm", false}, {src.wq, &dst.wq, "wq", false},
      {src.wk, &dst.wk, "wk", is_base},                   {src.wv, &dst.wv, "wv", is_base},
      {src.wo, &dst.wo, "wo", false},                     {src.ffn_norm, &dst.ffn_norm, "ffn_norm", false},
      {src.w_gate, &dst.w_gate, "w_gate", false},         {src.w_up, &dst.w_up, "w_up", false},
      {src.w_down, &dst.w_down, "w_down", false},         {src.q_norm, &dst.q_norm, "q_norm", true},
      {src.k_norm, &dst.k_norm, "k_norm", true}};
  for (auto& e : f) {
    e.v->assign(m.n_layers, nullptr);
    if (!e.p) {
      if (e.optional) continue;
      return fail(KVP_ERR_NULL, "%s.%s is NULL", name, e.n);
    }
    for (int l = 0; l < m.n_layers; ++l) {
      if (!e.p[l] && !e.optional) return fail(KVP_ERR_NULL, "%s.%s[%d] is NULL", name, e.n, l);
      if (!aligned16(e.p[l])) return fail(KVP_ERR_BAD_CONFIG, "%s.%s[%d] is not 16-byte aligned", name, e.n, l);
      (*e.v)[l] = e.p[l];
    }
  }
  // query / key normalisation is a trait of the whole stack: gains for every layer or for none;
  // the auxiliary stack needs both (its keys are what the predictor reads), the base stack's
  // key gains are read only by ordinary inference and by the generation loop
  for (int l = 0; l < m.n_layers; ++l) {
    if ((dst.q_norm[l] != nullptr) != (dst.q_norm[0] != nullptr) || (dst.k_norm[l] != nullptr) != (dst.k_norm[0] != nullptr))
      return fail(KVP_ERR_NULL, "%s.q_norm / k_norm: given for some layers only", name);
  }
  if (dst.k_norm[0] && !dst.q_norm[0]) return fail(KVP_ERR_NULL, "%s.k_norm given without q_norm", name);
  if (!is_base && dst.q_norm[0] && !dst.k_norm[0]) return fail(KVP_ERR_NULL, "%s.q_norm given without k_norm", name);
  return KVP_OK;
}

}  // namespace

namespace kvp {
const std::vector<const void*>& handle_pred_wk(const kvp_handle* h) { return h->pred_wk; }
const std::vector<const void*>& handle_pred_wv(const kvp_handle* h) { return h->pred_wv; }
const std::vector<int32_t>& handle_layer_map(const kvp_handle* h) { return h->layer_map; }
const kvp_config& handle_cfg(const kvp_handle* h) { return h->cfg; }
}  // namespace kvp

extern "C" {

const char* kvp_last_error(void) { return g_err; }
const char* kvp_version(void) { return "libkvp 0.1 (gfx950)"; }

// Host half of kvp_load_weights: validates the configuration and fills the handle's host-side plan
// (shapes, per-layer widths, layer map, kernel family).  Touches no device; kvp_debug_plan uses it alone.
static int init_host(const kvp_config* cfg, kvp_handle** out) {
  *out = nullptr;
  if (!cfg->layer_map) return fail(KVP_ERR_NULL, "layer_map is NULL");
  int rc;
  if ((rc = check_shape("base", cfg->base)) != KVP_OK) return rc;
  if ((rc = check_shape("aux", cfg->aux)) != KVP_OK) return rc;
  if (cfg->vocab < 1) return fail(KVP_ERR_BAD_CONFIG, "vocab < 1");
  if (cfg->dtype != KVP_DTYPE_F32 && cfg->dtype != KVP_DTYPE_BF16) return fail(KVP_ERR_BAD_CONFIG, "unknown dtype %d", cfg->dtype);
  if (cfg->max_batch < 1 || cfg->max_seq < 1) return fail(KVP_ERR_BAD_CONFIG, "max_batch / max_seq < 1");
  if ((int64_t)cfg->max_batch * cfg->max_seq > (int64_t)1 << 30) return fail(KVP_ERR_BAD_CONFIG, "max_batch * max_seq > 2^30");
  if (!(cfg->rope_theta > 0.f) || !(cfg->rms_eps >= 0.f)) return fail(KVP_ERR_BAD_CONFIG, "rope_theta must be > 0 and rms_eps >= 0");
  for (int i = 0; i < cfg->base.n_layers; ++i)
    if (cfg->layer_map[i] < 0 || cfg->layer_map[i] >= cfg->aux.n_layers)
      return fail(KVP_ERR_BAD_CONFIG, "layer_map[%d] = %d outside [0, %d)", i, cfg->layer_map[i], cfg->aux.n_layers);
  if (!cfg->base.layer_n_q_heads && !decode_attn_supported(cfg->base.head_dim, cfg->base.n_q_heads / cfg->base.n_kv_heads))
    return fail(KVP_ERR_BAD_CONFIG, "base: head_dim must be 16/32/64/128 and n_q/n_kv one of 1,2,3,4,6,8");
  kvp_handle* h = new (std::nothrow) kvp_handle();
  if (!h) return fail(KVP_ERR_HIP, "out of host memory");
  h->cfg = *cfg;
  h->layer_map.assign(cfg->layer_map, cfg->layer_map + cfg->base.n_layers);
  h->cfg.layer_map = h->layer_map.data();
  h->esize = cfg->dtype == KVP_DTYPE_F32 ? 4 : 2;
  if ((rc = copy_widths("base", cfg->base, true, h->b_nq, h->b_nkv, h->b_f)) != KVP_OK ||
      (rc = copy_widths("aux", cfg->aux, false, h->a_nq, h->a_nkv, h->a_f)) != KVP_OK) {
    delete h;
    return rc;
  }
  // the caller's width arrays were copied; the handle's configuration keeps the maxima only
  h->cfg.base.layer_n_q_heads = h->cfg.base.layer_n_kv_heads = h->cfg.base.layer_ffn_dim = nullptr;
  h->cfg.aux.layer_n_q_heads = h->cfg.aux.layer_n_kv_heads = h->cfg.aux.layer_ffn_dim = nullptr;
  const char* force = getenv("KVP_FORCE_GENERIC");
  h->force_generic = force && force[0] == '1';
  h->use_mfma = stack_mfma(h, h->cfg.aux);
  const char* pm = getenv("KVP_PRED_MAIN");            // "0" / "1": which stream runs the predictor (tuning override)
  h->pred_main = pm ? (pm[0] == '1' ? 1 : 0) : -1;
  *out = h;
  return KVP_OK;
}

int kvp_load_weights(const kvp_config* cfg, const kvp_weights* wts, kvp_handle** out) {
  if (out) *out = nullptr;
  if (!cfg || !wts || !out) return fail(KVP_ERR_NULL, "kvp_load_weights: NULL argument");
  kvp_handle* h = nullptr;
  int rc = init_host(cfg, &h);
  if (rc != KVP_OK) return rc;
  if (!wts->pred_wk || !wts->pred_wv) { delete h; return fail(KVP_ERR_NULL, "pred_wk / pred_wv is NULL"); }
  if ((rc = copy_model("base", cfg->base, wts->base, h->base, true)) != KVP_OK ||
      (rc = copy_model("aux", cfg->aux, wts->aux, h->aux, false)) != KVP_OK) {
    delete h;
    return rc;
  }
  for (int i = 0; i < cfg->base.n_layers; ++i) {
    if (!wts->pred_wk[i] || !wts->pred_wv[i]) { delete h; return fail(KVP_ERR_NULL, "pred_wk/pred_wv[%d] is NULL", i); }
    if (!aligned16(wts->pred_wk[i]) || !aligned16(wts->pred_wv[i])) {
      delete h;
      return fail(KVP_ERR_BAD_CONFIG, "pred_wk/pred_wv[%d] is not 16-byte aligned", i);
    }
    h->pred_wk.push_back(wts->pred_wk[i]);
    h->pred_wv.push_back(wts->pred_wv[i]);
  }

  // Device memory the handle owns: two rotary tables built once in double precision (max_seq x head_dim / 2
  // float2 each, a few MB), one flag word, and the predictor's pointer / layer-map tables (mfma_prepare).
  hipError_t e = hipGetDevice(&h->device);
  if (e != hipSuccess) { kvp_free(h); return fail(KVP_ERR_HIP, "hipGetDevice: %s", hipGetErrorString(e)); }
  size_t na = (size_t)cfg->max_seq * (cfg->aux.head_dim / 2), nb = (size_t)cfg->max_seq * (cfg->base.head_dim / 2);
  e = hipMalloc((void**)&h->rope_aux, na * sizeof(float2));
  if (e == hipSuccess) e = hipMalloc((void**)&h->rope_base, nb * sizeof(float2));
  if (e == hipSuccess) e = hipMalloc((void**)&h->flags, 256);
  if (e == hipSuccess) e = hipMemset(h->flags, 0, 256);
  if (e != hipSuccess) { kvp_free(h); return fail(KVP_ERR_HIP, "hipMalloc(rotary tables, flag word): %s", hipGetErrorString(e)); }
  launch_rope_table(h->rope_aux, cfg->max_seq, cfg->aux.head_dim / 2, (double)cfg->rope_theta, nullptr);
  launch_rope_table(h->rope_base, cfg->max_seq, cfg->base.head_dim / 2, (double)cfg->rope_theta, nullptr);
  e = hipDeviceSynchronize();
  if (e != hipSuccess) { kvp_free(h); return fail(KVP_ERR_HIP, "rotary table kernel: %s", hipGetErrorString(e)); }
  // address of the static scratch array on this device, for kvp_generation_step_static (which may not look it up itself)
  void* sp = nullptr;
  e = scratch_address(h->device, &sp);
  if (e != hipSuccess) { kvp_free(h); return fail(KVP_ERR_HIP, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e)); }
  const char* no_ov = getenv("KVP_NO_OVERLAP");
  if (h->use_mfma && !(no_ov && no_ov[0] == '1')) {
    // default priority, no implicit synchronisation with the legacy default stream
    bool ok = hipStreamCreateWithFlags(&h->side, hipStreamNonBlocking) == hipSuccess;
    ok = ok && hipEventCreateWithFlags(&h->ev_start, hipEventDisableTiming) == hipSuccess;
    ok = ok && hipEventCreateWithFlags(&h->ev_done, hipEventDisableTiming) == hipSuccess;
    h->ev_kv.assign(cfg->aux.n_layers, nullptr);
    for (int l = 0; ok && l < cfg->aux.n_layers; ++l)
      ok = hipEventCreateWithFlags(&h->ev_kv[l], hipEventDisableTiming) == hipSuccess;
    if (!ok) { kvp_free(h); return fail(KVP_ERR_HIP, "could not create the internal stream / events"); }
    h->overlap = true;
  }
  if (h->use_mfma && (rc = mfma_prepare(h, &h->mfma_tables)) != KVP_OK) {
    kvp_free(h);
    return fail(rc, "could not build the predictor's device tables");
  }
  *out = h;
  return KVP_OK;
}

int kvp_check_flags(kvp_handle* h, uint32_t* flags_out, int32_t clear) {
  if (!h || !flags_out) return fail(KVP_ERR_NULL, "kvp_check_flags: NULL argument");
  uint32_t v = 0;
  hipError_t e = hipMemcpy(&v, h->flags, sizeof(v), hipMemcpyDeviceToHost);
  if (e == hipSuccess && clear && v) e = hipMemset(h->flags, 0, sizeof(v));
  if (e != hipSuccess) return fail(KVP_ERR_HIP, "kvp_check_flags: %s", hipGetErrorString(e));
  *flags_out = v;
  return KVP_OK;
}

int kvp_debug_plan(const kvp_config* cfg, int32_t B, int32_t T, kvp_plan_region* regions, int32_t capacity,
                   int32_t* n_regions, uint64_t* total_bytes) {
  if (!cfg || !n_regions || !total_bytes) return fail(KVP_ERR_NULL, "kvp_debug_plan: NULL argument");
  kvp_handle* h = nullptr;
  int rc = init_host(cfg, &h);
  if (rc != KVP_OK) return rc;
  if (B < 1 || T < 1 || B > h->cfg.max_batch || T > h->cfg.max_seq) {
    delete h;
    return fail(KVP_ERR_BAD_SHAPE, "B = %d, T = %d outside [1, max_batch] x [1, max_seq]", B, T);
  }
  std::vector<PlanRegion> rs;
  Workspace w = plan_workspace(h, B, T, false, &rs);
  // What the launches of a B x T call touch in the split-partial region, from the launch-side split counts
  // (the planner sizes the region from bounds of its own; the two must agree for every shape).
  size_t part_touched = 0;
  for (int i = 0; i < h->cfg.base.n_layers; ++i) {
    size_t e = (size_t)decode_attn_splits(B, h->b_nkv[i], T) * B * h->b_nq[i] * (h->cfg.base.head_dim + kPartPad);
    if (e > part_touched) part_touched = e;
    const int Ka_i = h->a_nkv[h->layer_map[i]] * h->cfg.aux.head_dim;
    if (absorbed_attn_supported(Ka_i)) {
      e = (size_t)absorbed_splits(h, B, h->b_nq[i], Ka_i, T) * B * h->b_nq[i] * (Ka_i + kPartPad);
      if (e > part_touched) part_touched = e;
    }
  }
  *n_regions = (int32_t)rs.size();
  *total_bytes = w.total;
  for (int i = 0; regions && i < (int)rs.size() && i < capacity; ++i) {
    snprintf(regions[i].name, sizeof(regions[i].name), "%s", rs[i].name);
    regions[i].offset = rs[i].offset;
    regions[i].bytes = rs[i].bytes;
    regions[i].bytes_touched = strcmp(rs[i].name, "part") == 0 ? part_touched * sizeof(float) : rs[i].bytes;
  }
  delete h;
  return KVP_OK;
}

size_t kvp_workspace_bytes(const kvp_handle* h, int32_t B, int32_t T) {
  if (!h || B < 1 || T < 1 || B > h->cfg.max_batch || T > h->cfg.max_seq) return 0;
  return plan_workspace(h, B, T).total;
}

int kvp_aux_cache_offsets(const kvp_handle* h, int32_t B, int32_t T, size_t* k_offset, size_t* v_offset) {
  if (!h || !k_offset || !v_offset) return fail(KVP_ERR_NULL, "kvp_aux_cache_offsets: NULL argument");
  if (B < 1 || T < 1 || B > h->cfg.max_batch || T > h->cfg.max_seq) return fail(KVP_ERR_BAD_SHAPE, "B or T out of range");
  Workspace w = plan_workspace(h, B, T);
  *k_offset = w.aux_k;
  *v_offset = w.aux_v;
  return KVP_OK;
}

int kvp_run_stages(kvp_handle* h, uint32_t stages, const int32_t* tokens, int32_t B, int32_t T, void* k_cache,
                   void* v_cache, int64_t T_cap, float* logits, int32_t* argmax, void* workspace, size_t workspace_bytes,
                   void* hip_stream) {
  if (!h) return fail(KVP_ERR_NULL, "handle is NULL");
  const uint32_t known = KVP_STAGE_ALL | KVP_STAGE_BASE_ABSORBED, any_base = KVP_STAGE_BASE | KVP_STAGE_BASE_ABSORBED;
  if (!(stages & known) || (stages & ~known)) return fail(KVP_ERR_BAD_SHAPE, "bad stage mask 0x%x", stages);
  if ((stages & any_base) == any_base)
    return fail(KVP_ERR_BAD_SHAPE, "KVP_STAGE_BASE and KVP_STAGE_BASE_ABSORBED are two ways of running the same step: give one");
  if (!workspace) return fail(KVP_ERR_NULL, "workspace is NULL");
  if ((stages & (KVP_STAGE_AUX | any_base)) && !tokens) return fail(KVP_ERR_NULL, "tokens is NULL");
  if ((stages & (KVP_STAGE_PREDICT | KVP_STAGE_BASE)) && (!k_cache || !v_cache)) return fail(KVP_ERR_NULL, "k_cache / v_cache is NULL");
  if ((stages & any_base) && !logits && !argmax) return fail(KVP_ERR_NULL, "logits and argmax are both NULL");
  if (B < 1 || T < 1) return fail(KVP_ERR_BAD_SHAPE, "B = %d, T = %d must be >= 1", B, T);
  if (B > h->cfg.max_batch || T > h->cfg.max_seq)
    return fail(KVP_ERR_BAD_SHAPE, "B = %d, T = %d exceed max_batch = %d, max_seq = %d", B, T, h->cfg.max_batch, h->cfg.max_seq);
  if ((stages & (KVP_STAGE_PREDICT | KVP_STAGE_BASE)) && T_cap < T) return fail(KVP_ERR_BAD_SHAPE, "T_cap = %lld < T = %d", (long long)T_cap, T);
  if (((uintptr_t)workspace & 255) != 0) return fail(KVP_ERR_BAD_SHAPE, "workspace is not 256-byte aligned");
  if (!aligned16(k_cache) || !aligned16(v_cache) || !aligned16(logits) || ((uintptr_t)tokens & 3) || ((uintptr_t)argmax & 3))
    return fail(KVP_ERR_BAD_SHAPE, "k_cache / v_cache / logits must be 16-byte aligned, tokens / argmax 4-byte aligned");
  Workspace w = plan_workspace(h, B, T);
  if (workspace_bytes < w.total)
    return fail(KVP_ERR_WORKSPACE_TOO_SMALL, "workspace has %zu bytes, %zu needed", workspace_bytes, w.total);
  hipStream_t s = (hipStream_t)hip_stream;
  char* ws = (char*)workspace;
  if (h->cfg.dtype == KVP_DTYPE_F32)
    return run_stages<float>(h, stages, w, ws, tokens, B, T, k_cache, v_cache, T_cap, logits, argmax, s);
  return run_stages<bf16>(h, stages, w, ws, tokens, B, T, k_cache, v_cache, T_cap, logits, argmax, s);
}

int kvp_prefill_predict(kvp_handle* h, const int32_t* tokens, int32_t B, int32_t T, void* k_cache, void* v_cache,
                        int64_t T_cap, float* logits, int32_t* argmax, void* workspace, size_t workspace_bytes,
                        void* hip_stream) {
  return kvp_run_stages(h, KVP_STAGE_ALL, tokens, B, T, k_cache, v_cache, T_cap, logits, argmax, workspace,
                        workspace_bytes, hip_stream);
}

size_t kvp_reference_workspace_bytes(const kvp_handle* h, int32_t model, int32_t B, int32_t T) {
  if (!h || (model != KVP_MODEL_BASE && model != KVP_MODEL_AUX)) return 0;
  if (B < 1 || T < 1 || B > h->cfg.max_batch || T > h->cfg.max_seq) return 0;
  return plan_reference(h, model == KVP_MODEL_BASE ? h->cfg.base : h->cfg.aux, B, T).total;
}

int kvp_reference_prefill(kvp_handle* h, int32_t model, const int32_t* tokens, int32_t B, int32_t T, void* k_cache,
                          void* v_cache, int64_t T_cap, float* logits, int32_t* argmax, void* workspace,
                          size_t workspace_bytes, void* hip_stream) {
  if (!h) return fail(KVP_ERR_NULL, "handle is NULL");
  if (model != KVP_MODEL_BASE && model != KVP_MODEL_AUX) return fail(KVP_ERR_BAD_SHAPE, "model must be KVP_MODEL_BASE or KVP_MODEL_AUX");
  if (!tokens || !workspace) return fail(KVP_ERR_NULL, "tokens / workspace is NULL");
  if (!logits && !argmax) return fail(KVP_ERR_NULL, "logits and argmax are both NULL");
  if ((k_cache == nullptr) != (v_cache == nullptr)) return fail(KVP_ERR_NULL, "k_cache and v_cache must both be given or both be NULL");
  if (B < 1 || T < 1) return fail(KVP_ERR_BAD_SHAPE, "B = %d, T = %d must be >= 1", B, T);
  if (B > h->cfg.max_batch || T > h->cfg.max_seq)
    return fail(KVP_ERR_BAD_SHAPE, "B = %d, T = %d exceed max_batch = %d, max_seq = %d", B, T, h->cfg.max_batch, h->cfg.max_seq);
  if (k_cache && T_cap < T) return fail(KVP_ERR_BAD_SHAPE, "T_cap = %lld < T = %d", (long long)T_cap, T);
  if (((uintptr_t)workspace & 255) != 0) return fail(KVP_ERR_BAD_SHAPE, "workspace is not 256-byte aligned");
  if (!aligned16(k_cache) || !aligned16(v_cache) || !aligned16(logits) || ((uintptr_t)tokens & 3) || ((uintptr_t)argmax & 3))
    return fail(KVP_ERR_BAD_SHAPE, "k_cache / v_cache / logits must be 16-byte aligned, tokens / argmax 4-byte aligned");
  const bool is_base = model == KVP_MODEL_BASE;
  const kvp_model_shape& m = is_base ? h->cfg.base : h->cfg.aux;
  const ModelW& mw = is_base ? h->base : h->aux;
  if (!mw.final_norm || !mw.lm_head) return fail(KVP_ERR_NULL, "%s.final_norm / lm_head were not given to kvp_load_weights", is_base ? "base" : "aux");
  for (int l = 0; l < m.n_layers; ++l)
    if (!mw.wk[l] || !mw.wv[l]) return fail(KVP_ERR_NULL, "%s.wk / wv[%d] were not given to kvp_load_weights", is_base ? "base" : "aux", l);
  RefWorkspace r = plan_reference(h, m, B, T);
  if (workspace_bytes < r.total)
    return fail(KVP_ERR_WORKSPACE_TOO_SMALL, "workspace has %zu bytes, %zu needed", workspace_bytes, r.total);
  hipStream_t s = (hipStream_t)hip_stream;
  const float2* rope = is_base ? h->rope_base : h->rope_aux;
  if (h->cfg.dtype == KVP_DTYPE_F32)
    return run_reference<float>(h, m, mw, rope, r, (char*)workspace, tokens, B, T, k_cache, v_cache, T_cap, logits, argmax, s);
  return run_reference<bf16>(h, m, mw, rope, r, (char*)workspace, tokens, B, T, k_cache, v_cache, T_cap, logits, argmax, s);
}

size_t kvp_generation_workspace_bytes(const kvp_handle* h, int32_t B, int32_t T_total) {
  if (!h || B < 1 || T_total < 1 || B > h->cfg.max_batch || T_total > h->cfg.max_seq) return 0;
  return plan_workspace(h, B, T_total, true).total;
}

// Shared body of kvp_generation_step and kvp_generation_step_static: `scratch_bytes` of device scratch at
// `scratch_mem`, from the caller's workspace or from the library's static array.
static int generation_step(kvp_handle* h, const int32_t* tokens, int32_t B, int32_t pos, void* k_cache, void* v_cache,
                           int64_t T_cap, float* logits, int32_t* argmax, void* scratch_mem, size_t scratch_bytes,
                           const char* scratch_name, void* hip_stream) {
  if (!tokens || !k_cache || !v_cache) return fail(KVP_ERR_NULL, "tokens / caches is NULL");
  if (!logits && !argmax) return fail(KVP_ERR_NULL, "logits and argmax are both NULL");
  if (B < 1 || B > h->cfg.max_batch) return fail(KVP_ERR_BAD_SHAPE, "B = %d outside [1, max_batch = %d]", B, h->cfg.max_batch);
  if (pos < 1 || pos + 1 > h->cfg.max_seq) return fail(KVP_ERR_BAD_SHAPE, "pos = %d: pos + 1 must lie in [2, max_seq = %d]", pos, h->cfg.max_seq);
  if ((int64_t)pos + 1 > T_cap) return fail(KVP_ERR_BAD_SHAPE, "pos = %d does not fit T_cap = %lld", pos, (long long)T_cap);
  if (((uintptr_t)scratch_mem & 255) != 0) return fail(KVP_ERR_BAD_SHAPE, "%s is not 256-byte aligned", scratch_name);
  if (!aligned16(k_cache) || !aligned16(v_cache) || !aligned16(logits) || ((uintptr_t)tokens & 3) || ((uintptr_t)argmax & 3))
    return fail(KVP_ERR_BAD_SHAPE, "k_cache / v_cache / logits must be 16-byte aligned, tokens / argmax 4-byte aligned");
  for (int l = 0; l < h->cfg.base.n_layers; ++l) {
    if (!h->base.wk[l] || !h->base.wv[l]) return fail(KVP_ERR_NULL, "base.wk / wv[%d] were not given to kvp_load_weights", l);
    if (h->base.qk_norm() && !h->base.k_norm[l]) return fail(KVP_ERR_NULL, "base.k_norm[%d] was not given to kvp_load_weights", l);
  }
  Workspace w = plan_workspace(h, B, pos + 1, true);
  if (scratch_bytes < w.total)
    return fail(KVP_ERR_WORKSPACE_TOO_SMALL, "%s has %zu bytes, %zu needed", scratch_name, scratch_bytes, w.total);
  hipStream_t s = (hipStream_t)hip_stream;
  char* ws = (char*)scratch_mem;
  prof_mark(h, s, -1);
  int rc;
  if (h->cfg.dtype == KVP_DTYPE_F32)
    rc = run_base<float>(h, w, ws, tokens, B, 1, k_cache, v_cache, T_cap, logits, argmax, s, pos);
  else if (!h->force_generic)
    rc = run_base_bf16(h, w, ws, tokens, B, 1, k_cache, v_cache, T_cap, logits, argmax, s, pos);
  else
    rc = run_base<bf16>(h, w, ws, tokens, B, 1, k_cache, v_cache, T_cap, logits, argmax, s, pos);
  if (rc != KVP_OK) return rc;
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(KVP_ERR_HIP, "HIP error after launch: %s", hipGetErrorString(e));
  return KVP_OK;
}

int kvp_generation_step(kvp_handle* h, const int32_t* tokens, int32_t B, int32_t pos, void* k_cache, void* v_cache,
                        int64_t T_cap, float* logits, int32_t* argmax, void* workspace, size_t workspace_bytes,
                        void* hip_stream) {
  if (!h) return fail(KVP_ERR_NULL, "handle is NULL");
  if (!workspace) return fail(KVP_ERR_NULL, "workspace is NULL");
  return generation_step(h, tokens, B, pos, k_cache, v_cache, T_cap, logits, argmax, workspace, workspace_bytes, "workspace",
                         hip_stream);
}

size_t kvp_static_scratch_bytes(void) { return KVP_STATIC_SCRATCH_BYTES; }

int kvp_generation_step_static(kvp_handle* h, const int32_t* tokens, int32_t B, int32_t pos, void* k_cache, void* v_cache,
                               int64_t T_cap, float* logits, int32_t* argmax, void* hip_stream) {
  if (!h) return fail(KVP_ERR_NULL, "handle is NULL");
  if (h->prof_on) return fail(KVP_ERR_BAD_SHAPE, "kvp_generation_step_static: the per-class timers create events; disable them first");
  // The per-device address was looked up by kvp_load_weights; nothing is looked up or allocated here.
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev != h->device)
    return fail(KVP_ERR_BAD_CONFIG, "kvp_generation_step_static: current device %d is not the handle's device %d", dev, h->device);
  void* sp = nullptr;
  {
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    sp = g_scratch_ptr[dev];
  }
  if (!sp) return fail(KVP_ERR_HIP, "kvp_generation_step_static: the scratch array's address is unknown on device %d", dev);
  if (B >= 1 && B <= h->cfg.max_batch && pos >= 1 && pos + 1 <= h->cfg.max_seq) {
    const size_t need = plan_workspace(h, B, pos + 1, true).total;
    if (need > KVP_STATIC_SCRATCH_BYTES)
      return fail(KVP_ERR_WORKSPACE_TOO_SMALL, "kvp_generation_step_static: B = %d at %d cache entries needs %zu bytes of scratch, "
                  "the static array holds %zu; use kvp_generation_step with a workspace", B, pos + 1, need,
                  (size_t)KVP_STATIC_SCRATCH_BYTES);
  }
  return generation_step(h, tokens, B, pos, k_cache, v_cache, T_cap, logits, argmax, sp, KVP_STATIC_SCRATCH_BYTES,
                         "static scratch", hip_stream);
}

void kvp_debug_flash_guard(float limit) { mfma_set_flash_guard(limit); }

int kvp_profile_enable(kvp_handle* h, int32_t on) {
  if (!h) return fail(KVP_ERR_NULL, "handle is NULL");
  h->prof_on = on != 0;
  return KVP_OK;
}

static int prof_collect(kvp_handle* h) {
  for (size_t i = 0; i < h->prof_used; ++i) {
    ProfEvent& e = h->prof_pool[i];
    if (e.cls < 0 || i == 0) continue;
    hipError_t rc = hipEventSynchronize(e.ev);
    float ms = 0.f;
    if (rc == hipSuccess) rc = hipEventElapsedTime(&ms, h->prof_pool[i - 1].ev, e.ev);
    if (rc != hipSuccess) { h->prof_used = 0; return fail(KVP_ERR_HIP, "profile event: %s", hipGetErrorString(rc)); }
    h->prof_ms[e.cls] += ms;
    h->prof_n[e.cls] += 1;
  }
  h->prof_used = 0;
  return KVP_OK;
}

int kvp_profile_reset(kvp_handle* h) {
  if (!h) return fail(KVP_ERR_NULL, "handle is NULL");
  int rc = prof_collect(h);
  for (int i = 0; i < KVP_KC_COUNT; ++i) { h->prof_ms[i] = 0.0; h->prof_n[i] = 0; }
  return rc;
}

int kvp_profile_read(kvp_handle* h, double* ms, int64_t* launches) {
  if (!h || !ms || !launches) return fail(KVP_ERR_NULL, "kvp_profile_read: NULL argument");
  int rc = prof_collect(h);
  for (int i = 0; i < KVP_KC_COUNT; ++i) { ms[i] = h->prof_ms[i]; launches[i] = h->prof_n[i]; }
  return rc;
}

void kvp_free(kvp_handle* h) {
  if (!h) return;
  mfma_release(h->mfma_tables);
  if (h->side) { (void)hipStreamSynchronize(h->side); (void)hipStreamDestroy(h->side); }
  if (h->ev_start) (void)hipEventDestroy(h->ev_start);
  if (h->ev_done) (void)hipEventDestroy(h->ev_done);
  for (hipEvent_t e : h->ev_kv) if (e) (void)hipEventDestroy(e);
  if (h->rope_aux) (void)hipFree(h->rope_aux);
  if (h->rope_base) (void)hipFree(h->rope_base);
  if (h->flags) (void)hipFree(h->flags);
  for (auto& e : h->prof_pool) (void)hipEventDestroy(e.ev);
  delete h;
}

}  // extern "C"
