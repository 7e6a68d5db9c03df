// C-ABI layer of the LayerPipe hot path: argument checking, workspace layout, the gradient rings
// that realise the delay elements of Eq. 6, and the stream/event graph of one training step.
// All arithmetic lives in the HIP kernels behind lp_kernels.h; nothing here computes on the host.
#include "../../include/lp.h"
#include "../../include/lp_measure.h"

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <memory>
#include <new>
#include <string>
#include <unordered_map>
#include <vector>

#include "lp_kernels.h"

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

struct Layer {
  lp_layer_desc d;
  size_t n_params = 0;
  size_t in_elems = 0, z_elems = 0, a_elems = 0;  // whole batch
  int in_feat = 0, out_feat = 0;                  // per-sample flattened sizes
  size_t off_master = 0, off_work[2] = {0, 0}, off_ring = 0;
  size_t off_A[2] = {0, 0}, off_Z[2] = {0, 0};   // stashes; [1] differs from [0] only with forward run-ahead
  size_t off_dA = 0, off_dY = 0;
  bool has_A = false, has_Z = false, has_dA = false;
  int ring_slots = 1;
  int delay = 0;       // active d_l
  bool factor_ring = false;   // the ring holds (A_{l-1}, dY_l) pairs instead of G_l; the update multiplies them itself
  size_t ring_x_bytes = 0, ring_slot_bytes = 0;
  // Retimed update (lp_set_retimed_update): the delay elements of Eq. 6 sit on the weights.  The G task applies its
  // gradient at once (master = all gradients so far applied) and writes the result's bf16 copy as a new version;
  // F and dX of step n read version n - 1 - d_l.  There is no gradient ring and no update task.
  bool retimed = false;
  int n_versions = 0;          // d_l + 2 (a power of two with graph replay)
  size_t off_versions = 0, version_bytes = 0;
  int split_cols = 0;  // last columns of dA_{l-1} computed as a second, independent kernel (delta'')
  int cur = 0;         // working-weight buffer F and dX read now
  bool weights_set = false;
};

std::string g_create_error;

}  // namespace

struct lp_ctx {
  std::vector<Layer> layers;
  int L = 0, batch = 0, dtype = 0, loss = 0;
  float lr = 0.f;
  size_t ws_bytes = 0;
  size_t off_partials = 0, off_conv_scratch = 0;
  // split-K partial sums: [0] F and dX column ranges that start at column 0, [1] dW, [2] dX column
  // ranges that start elsewhere (delta' next to delta'' on another stream), [3] F on the forward
  // stream of a run-ahead step (next to the dX of the step before)
  size_t off_splitk[4] = {0, 0, 0, 0}, splitk_bytes[4] = {0, 0, 0, 0};
  bool run_ahead = false;
  // HIP-graph replay of whole steps (lp_set_graphs)
  struct GraphEntry { std::string key; hipGraph_t graph; hipGraphExec_t exec; };
  bool graphs = false;
  int graph_period = 2;              // steps after which every buffer choice of a step repeats
  std::vector<GraphEntry> graph_cache;
  long graph_captured = 0, graph_replayed = 0, graph_eager = 0;
  char* ws = nullptr;
  const void* gelu_lut = nullptr;   // GELU over all bf16 inputs (lp::gelu_lut_bf16), looked up by the F epilogue of GELU layers
  const float* gelu_grad_lut = nullptr;   // its derivative (lp::gelu_grad_lut_f32), looked up by the Hadamard product
  bool fuse_hadamard = true;        // lp_step folds f'(S_{l-1}) (.) into the epilogue of dX_l where the pair of layers allows it
  long n = 0;
  std::string err;
  bool events_ready = false;
  std::vector<hipEvent_t> ev_dy, ev_dx, ev_dw, ev_split, ev_upd;
  hipEvent_t ev_fork = nullptr, ev_join_w = nullptr, ev_join_u = nullptr;
  hipEvent_t ev_loss[2] = {nullptr, nullptr}, ev_bdone[2] = {nullptr, nullptr};
  std::vector<hipStream_t> streams_seen;
  // Bookkeeping that lets lp_step drop waits that earlier waits already imply (a wait that is followed
  // by a launch costs the host several times what the launch costs).  Every record on a stream gets that
  // stream's next sequence number; a stream that has waited for record q of stream s has thereby waited
  // for every earlier record of s.
  struct EvInfo { int src = -1; long seq = 0; };
  std::unordered_map<hipEvent_t, EvInfo> ev_info;
  std::vector<long> rec_count;                 // [stream index]: records so far
  std::vector<std::vector<long>> waited_seq;   // [waiting stream][recording stream]: newest record waited for
  // measurement aid (lp_profile)
  struct ProfRec { int task, layer; hipEvent_t e0, e1; };
  bool prof_on = false;
  std::vector<ProfRec> prof_recs;
  std::vector<hipEvent_t> prof_free;
  std::vector<double> prof_ms;   // [task * (L + 1) + layer], layer 0 = not tied to a layer (loss)
  std::vector<long> prof_n;
};

namespace {

int fail(lp_ctx* c, int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof(buf), fmt, ap);
  va_end(ap);
  if (c) c->err = buf; else g_create_error = buf;
  return code;
}
int fail_hip(lp_ctx* c, hipError_t e, const char* what) {
  return fail(c, LP_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}
#define LP_HIP(c, call)                                   \
  do {                                                    \
    hipError_t e__ = (call);                              \
    if (e__ != hipSuccess) return fail_hip(c, e__, #call); \
  } while (0)

// Runs the body of an entry point; a C++ exception (host memory exhausted in a container of the context) ends
// the call with LP_ERR_STATE instead of crossing the C boundary.
template <class Body>
int guarded(lp_ctx* c, const char* where, Body&& body) noexcept {
  try {
    return body();
  } catch (...) {
    try {
      if (c) { c->err = where; c->err += ": out of host memory or internal error"; }
      else { g_create_error = where; g_create_error += ": out of host memory or internal error"; }
    } catch (...) {
    }
    return LP_ERR_STATE;
  }
}

inline bool is_bf16(const lp_ctx* c) { return c->dtype == LP_BF16; }
inline size_t esize(const lp_ctx* c) { return is_bf16(c) ? 2 : 4; }
inline void note_stream(lp_ctx* c, hipStream_t s) {
  for (hipStream_t t : c->streams_seen)
    if (t == s) return;
  c->streams_seen.push_back(s);
}

inline int stream_index(lp_ctx* c, hipStream_t s) {
  for (size_t i = 0; i < c->streams_seen.size(); ++i)
    if (c->streams_seen[i] == s) return (int)i;
  c->streams_seen.push_back(s);
  return (int)c->streams_seen.size() - 1;
}
hipError_t record_on(lp_ctx* c, hipEvent_t e, hipStream_t s) {
  const int si = stream_index(c, s);
  if ((int)c->rec_count.size() <= si) c->rec_count.resize(si + 1, 0);
  lp_ctx::EvInfo& info = c->ev_info[e];
  info.src = si;
  info.seq = ++c->rec_count[si];
  return hipEventRecord(e, s);
}
// s waits for the latest record of e, unless that is implied: e was never recorded, was recorded on s
// itself (a stream runs in order), or s has already waited for that record or a later one of the same stream.
hipError_t wait_on(lp_ctx* c, hipStream_t s, hipEvent_t e) {
  auto it = c->ev_info.find(e);
  if (it == c->ev_info.end() || it->second.src < 0) return hipSuccess;
  const int di = stream_index(c, s), si = it->second.src;
  if (di == si) return hipSuccess;
  if ((int)c->waited_seq.size() <= di) c->waited_seq.resize(di + 1);
  std::vector<long>& w = c->waited_seq[di];
  if ((int)w.size() <= si) w.resize(si + 1, 0);
  if (w[si] >= it->second.seq) return hipSuccess;
  w[si] = it->second.seq;
  return hipStreamWaitEvent(s, e, 0);
}

// Brackets one task launch with timing events on its stream when profiling is on.
struct ProfScope {
  lp_ctx* c;
  hipStream_t s;
  hipEvent_t e1 = nullptr;
  ProfScope(lp_ctx* c_, int task, int layer, hipStream_t s_) : c(c_), s(s_) {
    if (!c->prof_on) return;
    hipEvent_t ev[2] = {nullptr, nullptr};
    for (hipEvent_t& e : ev) {
      if (!c->prof_free.empty()) { e = c->prof_free.back(); c->prof_free.pop_back(); }
      else if (hipEventCreate(&e) != hipSuccess) { e = nullptr; }
    }
    if (!ev[0] || !ev[1]) {
      for (hipEvent_t e : ev) if (e) c->prof_free.push_back(e);
      return;
    }
    (void)hipEventRecord(ev[0], s);
    e1 = ev[1];
    c->prof_recs.push_back({task, layer, ev[0], ev[1]});
  }
  ~ProfScope() {
    if (e1) (void)hipEventRecord(e1, s);
  }
};

int check_layer(lp_ctx* c, int l) {
  if (l < 1 || l > c->L) return fail(c, LP_ERR_LAYER, "layer index %d outside 1..%d", l, c->L);
  return LP_OK;
}
int need_ws(lp_ctx* c) {
  if (!c->ws) return fail(c, LP_ERR_STATE, "no workspace bound (call lp_bind_workspace)");
  return LP_OK;
}
int need_weights(lp_ctx* c, int l) {
  if (int r = need_ws(c)) return r;
  if (!c->layers[l - 1].weights_set) return fail(c, LP_ERR_STATE, "weights of layer %d were never set", l);
  return LP_OK;
}

inline int layer_no(const lp_ctx* c, const Layer& ly) { return (int)(&ly - c->layers.data()) + 1; }
// Version v of a retimed layer's working weights (v gradients applied).
inline void* version_slot(lp_ctx* c, const Layer& ly, long v) {
  return c->ws + ly.off_versions + (size_t)(v % ly.n_versions) * ly.version_bytes;
}
// The weights that the tasks of step c->n + 1 read.
inline void* work_w(lp_ctx* c, Layer& ly) {
  if (ly.retimed) { const long v = c->n - ly.d.delay; return version_slot(c, ly, v > 0 ? v : 0); }
  return is_bf16(c) ? (void*)(c->ws + ly.off_work[ly.cur]) : (void*)(c->ws + ly.off_master);
}
inline float* ring_slot(lp_ctx* c, Layer& ly, long step) {
  return (float*)(c->ws + ly.off_ring) + (size_t)(step % ly.ring_slots) * ly.n_params;
}
inline lp::ConvDesc conv_desc(const lp_ctx* c, const Layer& ly) {
  lp::ConvDesc cd;
  cd.B = c->batch; cd.H = ly.d.H; cd.W = ly.d.W; cd.Cin = ly.d.in; cd.Cout = ly.d.out;
  return cd;
}

// ---- the tasks, shared by the per-layer entry points and lp_step -------------------------------
// sk: which split-K scratch region a linear layer's product may use
hipError_t do_forward(lp_ctx* c, Layer& ly, const void* X, void* Z, void* A, hipStream_t s, int sk = 0) {
  ProfScope prof(c, LP_TASK_F, layer_no(c, ly), s);
  if (ly.d.kind == LP_LINEAR) {
    lp::GemmDesc g;
    g.A = X; g.B = work_w(c, ly);
    g.M = c->batch; g.N = ly.d.out; g.K = ly.d.in;
    g.lda = ly.d.in; g.ldb = ly.d.out; g.ldc = ly.d.out;
    g.a_kcontig = true; g.b_kcontig = false;
    g.out_z = Z; g.out_a = A; g.act = ly.d.act;
    g.act_lut = c->gelu_lut;
    g.splitk_scratch = (float*)(c->ws + c->off_splitk[sk]); g.splitk_bytes = c->splitk_bytes[sk];
    return is_bf16(c) ? lp::launch_gemm_bf16(g, s) : lp::launch_gemm_f32(g, s);
  }
  const lp::ConvDesc cd = conv_desc(c, ly);
  if (ly.d.pool == 2) {
    bool pooled = false;
    hipError_t e = lp::launch_conv_fwd(cd, is_bf16(c), X, work_w(c, ly), Z, nullptr, ly.d.act, s, A, &pooled);
    if (e != hipSuccess || !A || pooled) return e;
    return lp::launch_relu_pool(is_bf16(c), Z, A, c->batch, ly.d.H, ly.d.W, ly.d.out, ly.d.act, s);
  }
  return lp::launch_conv_fwd(cd, is_bf16(c), X, work_w(c, ly), Z, A, ly.d.act, s);
}

// had_of/S: the preceding layer and its stash when its Hadamard product (Eq. 3) rides in this product's epilogue
// (hadamard_fused); dX then receives dY_{l-1} and dA_{l-1} is never stored.
hipError_t do_grad_act(lp_ctx* c, Layer& ly, const void* dY, void* dX, int c0, int c1, hipStream_t s, const Layer* had_of = nullptr,
                       const void* S = nullptr) {
  ProfScope prof(c, LP_TASK_DX, layer_no(c, ly), s);
  if (had_of && (!is_bf16(c) || !S)) return hipErrorInvalidValue;
  const float* had_lut = had_of && had_of->d.act == LP_ACT_GELU ? c->gelu_grad_lut : nullptr;
  if (ly.d.kind == LP_LINEAR) {
    lp::GemmDesc g;
    const size_t es = esize(c);
    g.A = dY; g.B = (const char*)work_w(c, ly) + (size_t)c0 * ly.d.out * es;
    g.M = c->batch; g.N = c1 - c0; g.K = ly.d.out;
    g.lda = ly.d.out; g.ldb = ly.d.out; g.ldc = ly.d.in;
    g.a_kcontig = true; g.b_kcontig = true;
    g.out_z = (char*)dX + (size_t)c0 * es;
    if (had_of) {
      g.had_s = (const char*)S + (size_t)c0 * es;
      g.had_lut = had_lut;
    }
    // K is cut as for the whole product, whatever the column range: the split changes no bits
    const int sk = c0 == 0 ? 0 : 2;
    g.splitk_splits = lp::gemm_bf16_splitk_splits(c->batch, ly.d.in, ly.d.out);
    g.splitk_scratch = (float*)(c->ws + c->off_splitk[sk]); g.splitk_bytes = c->splitk_bytes[sk];
    return is_bf16(c) ? lp::launch_gemm_bf16(g, s) : lp::launch_gemm_f32(g, s);
  }
  const bool pooled_below = had_of && had_of->d.kind == LP_CONV3X3 && had_of->d.pool == 2;
  return lp::launch_conv_grad_act(conv_desc(c, ly), is_bf16(c), dY, work_w(c, ly), dX, c0, c1, s, had_of ? S : nullptr, had_lut, pooled_below);
}

hipError_t do_grad_weight(lp_ctx* c, Layer& ly, const void* X, const void* dY, float* G, hipStream_t s) {
  ProfScope prof(c, LP_TASK_DW, layer_no(c, ly), s);
  if (ly.d.kind == LP_LINEAR) {
    lp::GemmDesc g;
    g.A = X; g.B = dY;
    g.M = ly.d.in; g.N = ly.d.out; g.K = c->batch;
    g.lda = ly.d.in; g.ldb = ly.d.out; g.ldc = ly.d.out;
    g.a_kcontig = false; g.b_kcontig = false;
    g.out_f32 = G;
    g.splitk_scratch = (float*)(c->ws + c->off_splitk[1]); g.splitk_bytes = c->splitk_bytes[1];
    return is_bf16(c) ? lp::launch_gemm_bf16(g, s) : lp::launch_gemm_f32(g, s);
  }
  return lp::launch_conv_grad_weight(conv_desc(c, ly), is_bf16(c), X, dY, G, (float*)(c->ws + c->off_conv_scratch), s);
}

hipError_t do_act_grad(lp_ctx* c, Layer& ly, const void* dA, const void* S, void* dY, hipStream_t s) {
  ProfScope prof(c, LP_TASK_HADAMARD, layer_no(c, ly), s);
  if (ly.d.kind == LP_CONV3X3 && ly.d.pool == 2)
    return lp::launch_act_grad_pool(is_bf16(c), ly.d.act, dA, S, dY, c->batch, ly.d.H, ly.d.W, ly.d.out, s);
  return lp::launch_act_grad(is_bf16(c), ly.d.act, dA, S, dY, ly.z_elems, s, is_bf16(c) ? c->gelu_grad_lut : nullptr);
}

// Whether lp_step applies the Hadamard product of layer `pv` inside the dX product of the layer `ly` above it
// (Sec. III-B moves that product next to the task that feeds it; here it shares its kernel): a bf16 context and an
// element-wise ReLU or GELU below (tanh / sigmoid keep the stand-alone kernel), or a 2 x 2 max-pooled ReLU
// convolution below a convolution, whose epilogue then also routes each gradient to its window's maximum.
// Same bits either way.
bool hadamard_fused(const lp_ctx* c, const Layer& ly, const Layer& pv) {
  if (!c->fuse_hadamard || !is_bf16(c)) return false;
  if (pv.d.kind == LP_CONV3X3 && pv.d.pool == 2) return ly.d.kind == LP_CONV3X3 && pv.d.act == LP_ACT_RELU && pv.has_Z;
  if (pv.off_dY == pv.off_dA) return false;   // identity: there is no product
  return pv.d.act == LP_ACT_RELU || (pv.d.act == LP_ACT_GELU && c->gelu_grad_lut != nullptr);
}

hipError_t do_loss(lp_ctx* c, const void* ZL, const void* target, void* dYL, float* loss_dev, hipStream_t s) {
  ProfScope prof(c, LP_TASK_LOSS, 0, s);
  const Layer& last = c->layers[c->L - 1];
  float* partials = (float*)(c->ws + c->off_partials);
  if (c->loss == LP_LOSS_SOFTMAX_CE)
    return lp::launch_softmax_ce(is_bf16(c), ZL, (const int*)target, dYL, loss_dev, partials, c->batch, last.out_feat, s);
  return lp::launch_mse(is_bf16(c), ZL, target, dYL, loss_dev, partials, c->batch, last.out_feat, s);
}

// The G task of step `step` as lp_step runs it: the product into its ring slot, or, for a layer with a
// factor ring, only a copy of the two factors (the product is left to the delayed update).
hipError_t enqueue_G(lp_ctx* c, Layer& ly, const void* X, const void* dY, long step, hipStream_t s) {
  if (ly.retimed) {
    // Eq. 6 retimed: G_l(step) is applied to the master weights tile by tile as the product leaves the accumulators
    // (SgdEpilogue: the arithmetic of sgd_kernel) and the bf16 copy of the result becomes version `step`, which
    // the steps from step + d_l + 1 on read.  Same product kernel and summation order as lp_grad_weight (a convolution
    // applies the update where it sums its split-K partials).
    ProfScope prof(c, LP_TASK_DW, layer_no(c, ly), s);
    if (ly.d.kind == LP_CONV3X3)
      return lp::launch_conv_grad_weight(conv_desc(c, ly), true, X, dY, nullptr, (float*)(c->ws + c->off_conv_scratch), s,
                                         (float*)(c->ws + ly.off_master), version_slot(c, ly, step), c->lr);
    lp::GemmDesc g;
    g.A = X; g.B = dY;
    g.M = ly.d.in; g.N = ly.d.out; g.K = c->batch;
    g.lda = ly.d.in; g.ldb = ly.d.out; g.ldc = ly.d.out;
    g.a_kcontig = false; g.b_kcontig = false;
    g.out_z = version_slot(c, ly, step);
    g.sgd_master = (float*)(c->ws + ly.off_master);
    g.sgd_lr = c->lr;
    // K is cut where lp_grad_weight cuts it (same scratch region, same rule), and the kernel that adds the partial sums applies the update
    g.splitk_scratch = (float*)(c->ws + c->off_splitk[1]); g.splitk_bytes = c->splitk_bytes[1];
    return lp::launch_gemm_bf16(g, s);
  }
  if (!ly.factor_ring) return do_grad_weight(c, ly, X, dY, ring_slot(c, ly, step), s);
  ProfScope prof(c, LP_TASK_DW, layer_no(c, ly), s);
  char* slot = c->ws + ly.off_ring + (size_t)(step % ly.ring_slots) * ly.ring_slot_bytes;
  return lp::launch_copy2(X, slot, ly.in_elems * esize(c), dY, slot + ly.ring_x_bytes, ly.z_elems * esize(c), s);
}

// The delayed update with the gradient of step `src` (Eq. 6).  Factor ring: G_l(src) = A_{l-1}(src)^T . dY_l(src)
// is formed tile by tile from the stored factors by the same kernel that lp_grad_weight runs, and each
// tile is applied to the weights in its epilogue instead of being stored (same bits as the two-kernel path).
hipError_t do_update(lp_ctx* c, Layer& ly, const float* G, hipStream_t s);
hipError_t enqueue_update(lp_ctx* c, Layer& ly, long src, hipStream_t s) {
  if (!ly.factor_ring) return do_update(c, ly, ring_slot(c, ly, src), s);
  ProfScope prof(c, LP_TASK_UPDATE, layer_no(c, ly), s);
  const char* slot = c->ws + ly.off_ring + (size_t)(src % ly.ring_slots) * ly.ring_slot_bytes;
  lp::GemmDesc g;
  g.A = slot; g.B = slot + ly.ring_x_bytes;
  g.M = ly.d.in; g.N = ly.d.out; g.K = c->batch;
  g.lda = ly.d.in; g.ldb = ly.d.out; g.ldc = ly.d.out;
  g.a_kcontig = false; g.b_kcontig = false;
  g.out_z = c->ws + ly.off_work[ly.cur ^ 1];
  g.sgd_master = (float*)(c->ws + ly.off_master);
  g.sgd_lr = c->lr;
  return lp::launch_gemm_bf16(g, s);
}

// Applies W <- W - lr*G; BF16 writes the other working buffer.  Does not flip `cur`.
hipError_t do_update(lp_ctx* c, Layer& ly, const float* G, hipStream_t s) {
  ProfScope prof(c, LP_TASK_UPDATE, layer_no(c, ly), s);
  float* master = (float*)(c->ws + ly.off_master);
  void* work_out = is_bf16(c) ? (void*)(c->ws + ly.off_work[ly.cur ^ 1]) : nullptr;
  return lp::launch_sgd(master, G, work_out, c->lr, ly.n_params, s);
}

int ensure_events(lp_ctx* c) {
  if (c->events_ready) return LP_OK;
  auto mk = [&](hipEvent_t* e) { return hipEventCreateWithFlags(e, hipEventDisableTiming); };
  c->ev_dy.assign(c->L, nullptr);
  c->ev_dx.assign(c->L, nullptr);
  c->ev_dw.assign(c->L, nullptr);
  c->ev_split.assign(c->L, nullptr);
  c->ev_upd.assign(c->L, nullptr);
  for (int l = 0; l < c->L; ++l) {
    LP_HIP(c, mk(&c->ev_split[l]));
    LP_HIP(c, mk(&c->ev_upd[l]));
    LP_HIP(c, mk(&c->ev_dy[l]));
    LP_HIP(c, mk(&c->ev_dx[l]));
    LP_HIP(c, mk(&c->ev_dw[l]));
  }
  LP_HIP(c, mk(&c->ev_fork));
  LP_HIP(c, mk(&c->ev_join_w));
  LP_HIP(c, mk(&c->ev_join_u));
  for (int p = 0; p < 2; ++p) { LP_HIP(c, mk(&c->ev_loss[p])); LP_HIP(c, mk(&c->ev_bdone[p])); }
  c->events_ready = true;
  return LP_OK;
}

// Offsets of everything the context keeps in the caller's workspace.  Depends on the layer table and
// on whether forward run-ahead is enabled (two stashes per layer then).
void layout_workspace(lp_ctx* c) {
  const int L = c->L;
  const size_t es = esize(c);
  for (size_t& b : c->splitk_bytes) b = 0;
  c->graph_period = 2;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes); return o; };
  size_t conv_scratch = 0;
  for (int i = 0; i < L; ++i) {
    Layer& ly = c->layers[i];
    const bool last = i == L - 1;
    const bool pooled = ly.d.kind == LP_CONV3X3 && ly.d.pool == 2;
    ly.off_master = take(ly.n_params * 4);
    if (c->dtype == LP_BF16 && !ly.retimed) { ly.off_work[0] = take(ly.n_params * 2); ly.off_work[1] = take(ly.n_params * 2); }
    // d_l + 1 slots; with graph replay rounded up to a power of two, so that the slot a step uses repeats
    // with a short common period
    ly.ring_slots = ly.d.delay + 1;
    if (c->graphs) { int r = 1; while (r < ly.ring_slots) r *= 2; ly.ring_slots = r; }
    if (ly.ring_slots > c->graph_period && !ly.retimed) c->graph_period = ly.ring_slots;
    if (ly.retimed) {
      // d_l + 2 versions: step n writes version n while it (and, with run-ahead, F of step n + 1) still reads
      // versions n - 1 - d_l and n - d_l
      ly.n_versions = ly.d.delay + 2;
      if (c->graphs) { int r = 1; while (r < ly.n_versions) r *= 2; ly.n_versions = r; }
      if (ly.n_versions > c->graph_period) c->graph_period = ly.n_versions;
      ly.version_bytes = align_up(ly.n_params * 2);
      ly.off_versions = take((size_t)ly.n_versions * ly.version_bytes);
      ly.off_ring = 0;
    } else if (ly.factor_ring) {
      ly.ring_x_bytes = align_up(ly.in_elems * es);
      ly.ring_slot_bytes = ly.ring_x_bytes + align_up(ly.z_elems * es);
      ly.off_ring = take((size_t)ly.ring_slots * ly.ring_slot_bytes);
    } else {
      ly.off_ring = take((size_t)ly.ring_slots * ly.n_params * 4);
    }
    ly.has_A = !last;
    // the Hadamard factor is computed from Z; only ReLU's can be read off A (same sign)
    ly.has_Z = last || pooled || (ly.d.act != LP_ACT_RELU && ly.d.act != LP_ACT_IDENTITY);
    ly.has_dA = !last;
    for (int p = 0; p < 2; ++p) {
      if (p == 1 && !c->run_ahead) { ly.off_A[1] = ly.off_A[0]; ly.off_Z[1] = ly.off_Z[0]; break; }
      if (ly.has_A) ly.off_A[p] = take(ly.a_elems * es);
      if (ly.has_Z) ly.off_Z[p] = take(ly.z_elems * es);
    }
    if (ly.has_dA) ly.off_dA = take(ly.a_elems * es);
    // identity hidden layer without pool: delta equals dA, share the buffer
    if (ly.has_dA && ly.d.act == LP_ACT_IDENTITY && !pooled) ly.off_dY = ly.off_dA;
    else ly.off_dY = take(ly.z_elems * es);
    if (ly.d.kind == LP_CONV3X3) {
      size_t sc = lp::conv_grad_weight_scratch_bytes(conv_desc(c, ly));
      if (sc > conv_scratch) conv_scratch = sc;
    }
  }
  const Layer& lastl = c->layers[L - 1];
  c->off_partials = take(lp::loss_partials_count(c->loss == LP_LOSS_MSE, c->batch, lastl.out_feat) * 4);
  c->off_conv_scratch = take(conv_scratch);
  if (c->dtype == LP_BF16) {
    for (int i = 0; i < L; ++i) {
      const Layer& ly = c->layers[i];
      if (ly.d.kind != LP_LINEAR) continue;
      const size_t f = lp::gemm_bf16_splitk_bytes(c->batch, ly.d.out, ly.d.in), dx = lp::gemm_bf16_splitk_bytes(c->batch, ly.d.in, ly.d.out);
      const size_t dw = lp::gemm_bf16_splitk_bytes(ly.d.in, ly.d.out, c->batch);
      if (f > c->splitk_bytes[0]) c->splitk_bytes[0] = f;
      if (dx > c->splitk_bytes[0]) c->splitk_bytes[0] = dx;
      if (dx > c->splitk_bytes[2]) c->splitk_bytes[2] = dx;
      if (dw > c->splitk_bytes[1]) c->splitk_bytes[1] = dw;
      if (c->run_ahead && f > c->splitk_bytes[3]) c->splitk_bytes[3] = f;
    }
    for (int k = 0; k < 4; ++k) c->off_splitk[k] = take(c->splitk_bytes[k]);
  }
  c->ws_bytes = off;
}

// One training step with the forward pass on a stream of its own, so that F(n+1) overlaps the backward
// pass of step n wherever the delays allow it (Sec. III-A: the weights F_l(n+1) reads, W_l(n), need only
// G_l(n - d_l)).  The arithmetic of every task, and so every result, is that of the serial order; only
// the waits differ.  Streams: sF forward chain and loss, sC delta chain, sW G tasks, sU updates.
// There is no fork/join per step; each hazard has its own event (an event that was never recorded
// does not block, which covers the first steps):
//   stash A_l/Z_l[n&1]  written by F_l(n), read by G_{l+1}(n) and the Hadamard of layer l in B(n):
//                       F(n+2) waits for the end of B(n) (ev_bdone[n&1])
//   working weights     F_l(n+1) waits for update_l(n) (ev_upd[l]); update_l(n+1) overwrites the copy
//                       that F_l(n) and dX_l(n) read: it waits for dX_l(n) (layer 1: for the loss of step n)
//   gradient ring       update_l(n) waits for the newest G_l (ev_dw[l]); G_l(n) overwrites the slot
//                       update_l(n-1) read: it waits for ev_upd[l]
//   dY_L                written by the loss of step n+1: waits for dX_L(n) and G_L(n)
//   delta chain         B(n) starts at the loss of step n (ev_loss[n&1]); within B(n) as in the serial step,
//                       and sC ends each step by waiting for that step's G tasks, so dA/dY buffers are free
int step_run_ahead(lp_ctx* c, const void* X0, const void* target, float* loss_dev, void* const* streams) {
  hipStream_t sC = (hipStream_t)streams[0], sW = (hipStream_t)streams[1], sU = (hipStream_t)streams[2], sF = (hipStream_t)streams[3];
  for (hipStream_t s : {sC, sW, sU, sF}) note_stream(c, s);
  if (int r = ensure_events(c)) return r;
  const int L = c->L;
  const long n = c->n + 1;
  const int p = (int)(n & 1);
  std::vector<char> updated(L, 0);

  auto issue_update = [&](int i) -> int {
    Layer& ly = c->layers[i];
    const long src = n - ly.delay;
    if (src < 1) return LP_OK;
    LP_HIP(c, wait_on(c, sU, c->ev_dw[i]));                       // G_l(src) is in the ring
    LP_HIP(c, wait_on(c, sU, i > 0 ? c->ev_dx[i] : c->ev_loss[p ^ 1]));   // readers of the copy being overwritten
    LP_HIP(c, enqueue_update(c, ly, src, sU));
    LP_HIP(c, record_on(c, c->ev_upd[i], sU));
    updated[i] = 1;
    return LP_OK;
  };
  // forward chain of step n on sF
  LP_HIP(c, wait_on(c, sF, c->ev_bdone[p]));
  const void* a_prev = X0;
  for (int i = 0; i < L; ++i) {
    Layer& ly = c->layers[i];
    void* Z = ly.has_Z ? c->ws + ly.off_Z[p] : nullptr;
    void* A = ly.has_A ? c->ws + ly.off_A[p] : nullptr;
    // W_l(n-1) is complete (recorded by update_l(n-1) at the latest).  A retimed layer reads the version that the G
    // task of step n - 1 - d_l wrote: finished with B(n-2) for d_l > 0, else the newest G task
    if (!ly.retimed) LP_HIP(c, wait_on(c, sF, c->ev_upd[i]));
    else if (ly.d.delay == 0) LP_HIP(c, wait_on(c, sF, c->ev_dw[i]));
    LP_HIP(c, do_forward(c, ly, a_prev, Z, A, sF, 3));
    a_prev = A;
  }
  Layer& last = c->layers[L - 1];
  LP_HIP(c, wait_on(c, sF, c->ev_dx[L - 1]));
  LP_HIP(c, wait_on(c, sF, c->ev_dw[L - 1]));
  LP_HIP(c, do_loss(c, c->ws + last.off_Z[p], target, c->ws + last.off_dY, loss_dev, sF));
  LP_HIP(c, record_on(c, c->ev_loss[p], sF));

  // Updates that need no gradient of this step (their G tasks ran in earlier steps).  Enqueued after
  // the forward chain so that F_l(n) above waited for update_l(n-1), not for these.
  for (int i = L - 1; i >= 0; --i)
    if (c->layers[i].delay > 0 && !c->layers[i].retimed)
      if (int r = issue_update(i)) return r;

  // backward pass of step n
  LP_HIP(c, wait_on(c, sC, c->ev_loss[p]));
  LP_HIP(c, record_on(c, c->ev_dy[L - 1], sC));
  for (int i = L - 1; i >= 0; --i) {
    Layer& ly = c->layers[i];
    const void* x_in = i == 0 ? X0 : (const void*)(c->ws + c->layers[i - 1].off_A[p]);
    const void* dY = c->ws + ly.off_dY;
    if (i > 0) {
      Layer& pv = c->layers[i - 1];
      const void* S = pv.has_Z ? c->ws + pv.off_Z[p] : c->ws + pv.off_A[p];
      const bool fused = hadamard_fused(c, ly, pv);
      void* dX = c->ws + (fused ? pv.off_dY : pv.off_dA);
      const Layer* had = fused ? &pv : nullptr;
      if (ly.split_cols > 0) {
        const int cut = ly.d.in - ly.split_cols;
        LP_HIP(c, wait_on(c, sW, c->ev_dy[i]));
        LP_HIP(c, do_grad_act(c, ly, dY, dX, cut, ly.d.in, sW, had, S));
        LP_HIP(c, record_on(c, c->ev_split[i], sW));
        LP_HIP(c, do_grad_act(c, ly, dY, dX, 0, cut, sC, had, S));
        LP_HIP(c, wait_on(c, sC, c->ev_split[i]));
      } else {
        LP_HIP(c, do_grad_act(c, ly, dY, dX, 0, ly.d.in, sC, had, S));
      }
      LP_HIP(c, record_on(c, c->ev_dx[i], sC));
      if (pv.off_dY != pv.off_dA && !fused) LP_HIP(c, do_act_grad(c, pv, c->ws + pv.off_dA, S, c->ws + pv.off_dY, sC));
      LP_HIP(c, record_on(c, c->ev_dy[i - 1], sC));
    }
    LP_HIP(c, wait_on(c, sW, c->ev_dy[i]));
    // the ring slot's previous gradient has been applied.  (The version a retimed G task overwrites was last read by
    // F_l and dX_l of step n-1, which precede this step's delta chain on sC and therefore ev_dy above.)
    if (!ly.retimed) LP_HIP(c, wait_on(c, sW, c->ev_upd[i]));
    LP_HIP(c, enqueue_G(c, ly, x_in, dY, n, sW));
    LP_HIP(c, record_on(c, c->ev_dw[i], sW));
    if (!updated[i] && !ly.retimed)
      if (int r = issue_update(i)) return r;
  }
  LP_HIP(c, record_on(c, c->ev_join_w, sW));
  LP_HIP(c, wait_on(c, sC, c->ev_join_w));
  LP_HIP(c, record_on(c, c->ev_bdone[p], sC));

  for (int i = 0; i < L; ++i)
    if (updated[i]) c->layers[i].cur ^= 1;
  c->n = n;
  return LP_OK;
}

// Enqueues every task of step n = c->n + 1 in the serial-step order: one fork from sC at the start, one
// join into sC at the end, so the whole step is a single-entry, single-exit piece of work on sC (which
// is what lets it be captured into a graph).  Changes no host state; `updated` says which layers'
// working weights were rewritten.
constexpr long kChipTiles = 256;   // one 256 x 256 tile per CU
inline long tiles_256(int m, int n) { return (long)((m + 255) / 256) * ((n + 255) / 256); }

int enqueue_step(lp_ctx* c, const void* X0, const void* target, float* loss_dev, hipStream_t sC, hipStream_t sW, hipStream_t sU,
                 bool multi, std::vector<char>& updated) {
  const int L = c->L;
  const long n = c->n + 1;  // the step in progress
  const bool bf = is_bf16(c);
  updated.assign(L, 0);

  if (multi) {
    LP_HIP(c, record_on(c, c->ev_fork, sC));
    if (sW != sC) LP_HIP(c, wait_on(c, sW, c->ev_fork));
    if (sU != sC) LP_HIP(c, wait_on(c, sU, c->ev_fork));
  }

  // Delayed updates whose gradient is already in the ring (d_l > 0).  BF16 keeps two versions of
  // the working weights, so W_l(n) can be produced while this step still reads W_l(n-1).
  auto issue_update = [&](int i) -> int {
    Layer& ly = c->layers[i];
    const long src = n - ly.delay;
    if (src >= 1) {
      LP_HIP(c, enqueue_update(c, ly, src, sU));
      updated[i] = 1;
    }
    return LP_OK;
  };
  if (bf)
    for (int i = L - 1; i >= 0; --i)
      if (c->layers[i].delay > 0 && !c->layers[i].retimed)
        if (int r = issue_update(i)) return r;

  // forward chain
  const void* a_prev = X0;
  for (int i = 0; i < L; ++i) {
    Layer& ly = c->layers[i];
    void* Z = ly.has_Z ? c->ws + ly.off_Z[0] : nullptr;
    void* A = ly.has_A ? c->ws + ly.off_A[0] : nullptr;
    LP_HIP(c, do_forward(c, ly, a_prev, Z, A, sC));
    a_prev = A;
  }
  Layer& last = c->layers[L - 1];
  LP_HIP(c, do_loss(c, c->ws + last.off_Z[0], target, c->ws + last.off_dY, loss_dev, sC));
  if (multi) LP_HIP(c, record_on(c, c->ev_dy[L - 1], sC));

  // backward: the delta chain on sC first (critical loop), G on sW, updates on sU
  for (int i = L - 1; i >= 0; --i) {
    Layer& ly = c->layers[i];
    const void* x_in = i == 0 ? X0 : (const void*)(c->ws + c->layers[i - 1].off_A[0]);
    const void* dY = c->ws + ly.off_dY;
    if (i > 0) {
      Layer& pv = c->layers[i - 1];
      const void* S = pv.has_Z ? c->ws + pv.off_Z[0] : c->ws + pv.off_A[0];
      const bool fused = hadamard_fused(c, ly, pv);   // then dX_l writes dY_{l-1} itself
      void* dX = c->ws + (fused ? pv.off_dY : pv.off_dA);
      const Layer* had = fused ? &pv : nullptr;
      if (ly.split_cols > 0) {
        // delta' on the critical stream, delta'' (the columns the next stage borrowed, Sec. III-B) as an
        // independent kernel on the stream that otherwise carries the G tasks, ahead of this layer's G
        const int cut = ly.d.in - ly.split_cols;
        if (multi && sW != sC) LP_HIP(c, wait_on(c, sW, c->ev_dy[i]));
        LP_HIP(c, do_grad_act(c, ly, dY, dX, cut, ly.d.in, sW, had, S));
        if (multi && sW != sC) LP_HIP(c, record_on(c, c->ev_split[i], sW));
        LP_HIP(c, do_grad_act(c, ly, dY, dX, 0, cut, sC, had, S));
        if (multi && sW != sC) LP_HIP(c, wait_on(c, sC, c->ev_split[i]));
      } else {
        LP_HIP(c, do_grad_act(c, ly, dY, dX, 0, ly.d.in, sC, had, S));
      }
      if (multi && !bf) LP_HIP(c, record_on(c, c->ev_dx[i], sC));   // only an in-place (F32) update waits for it
      if (pv.off_dY != pv.off_dA && !fused) LP_HIP(c, do_act_grad(c, pv, c->ws + pv.off_dA, S, c->ws + pv.off_dY, sC));
      if (multi) LP_HIP(c, record_on(c, c->ev_dy[i - 1], sC));
    }
    // A G product that fills every CU with 256 x 256 tiles, next to a delta product that does so too, gains
    // nothing from a stream of its own: the two kernels only take turns on the CUs and break up each other's
    // L2 tile blocks.  It then follows dX_l on the critical stream; smaller products overlap on sW.
    const bool fills_chip = ly.d.kind == LP_LINEAR && !ly.factor_ring && tiles_256(ly.d.in, ly.d.out) >= kChipTiles &&
                            (i == 0 || tiles_256(c->batch, ly.d.in) >= kChipTiles);
    hipStream_t sG = fills_chip ? sC : sW;
    if (multi && sG != sC) LP_HIP(c, wait_on(c, sG, c->ev_dy[i]));
    LP_HIP(c, enqueue_G(c, ly, x_in, dY, n, sG));
    if (ly.retimed) continue;   // the G task has applied its gradient itself; nothing in this step reads what it wrote
    if (multi && !updated[i]) LP_HIP(c, record_on(c, c->ev_dw[i], sG));   // only this step's own update waits for it
    if (!updated[i]) {
      // d_l = 0 needs this step's G; an F32 context updates in place, so it also has to wait for
      // the last reader of W_l(n-1), which is dX_l (layer 1: the forward pass, long finished)
      if (multi) {
        if (ly.delay == 0 && sU != sG) LP_HIP(c, wait_on(c, sU, c->ev_dw[i]));
        if (!bf && sU != sC) LP_HIP(c, wait_on(c, sU, i > 0 ? c->ev_dx[i] : c->ev_dy[L - 1]));
      }
      if (int r = issue_update(i)) return r;
    }
  }

  if (multi) {
    if (sW != sC) { LP_HIP(c, record_on(c, c->ev_join_w, sW)); LP_HIP(c, wait_on(c, sC, c->ev_join_w)); }
    if (sU != sC) { LP_HIP(c, record_on(c, c->ev_join_u, sU)); LP_HIP(c, wait_on(c, sC, c->ev_join_u)); }
  }
  return LP_OK;
}

void drop_graphs(lp_ctx* c) {
  for (auto& g : c->graph_cache) {
    (void)hipGraphExecDestroy(g.exec);
    (void)hipGraphDestroy(g.graph);
  }
  c->graph_cache.clear();
}

constexpr size_t kMaxGraphs = 512;

// Runs step n = c->n + 1: eagerly, or (lp_set_graphs) as one graph launch on sC.  Every pointer a task
// of the step uses is a function of the key below: the ring slots and the stash-free serial layout
// repeat with c->graph_period, the working-weight copies with the layers' `cur` bits, the rest is the
// caller's.  A step is captured the first time its key is seen and replayed afterwards.  Steps inside
// the warm-up (some update still skipped) and profiled steps run eagerly.
int run_or_replay_step(lp_ctx* c, const void* X0, const void* target, float* loss_dev, hipStream_t sC, hipStream_t sW, hipStream_t sU,
                       bool multi, std::vector<char>& updated) {
  const long n = c->n + 1;
  long warm = 1;
  for (const Layer& ly : c->layers)
    if (ly.delay + 1 > warm) warm = ly.delay + 1;
  // the step after the warm-up still runs eagerly: by then every kernel has been launched once
  // outside a capture (first launches set function attributes)
  if (!c->graphs || c->prof_on || n <= warm + 1) {
    if (c->graphs) c->graph_eager += 1;
    return enqueue_step(c, X0, target, loss_dev, sC, sW, sU, multi, updated);
  }
  std::string key;
  auto put = [&](const void* p, size_t bytes) { key.append((const char*)p, bytes); };
  const long phase = n % c->graph_period;
  put(&phase, sizeof phase);
  put(&X0, sizeof X0); put(&target, sizeof target); put(&loss_dev, sizeof loss_dev);
  put(&sC, sizeof sC); put(&sW, sizeof sW); put(&sU, sizeof sU);
  for (const Layer& ly : c->layers) { put(&ly.cur, sizeof ly.cur); put(&ly.delay, sizeof ly.delay); put(&ly.split_cols, sizeof ly.split_cols); }

  updated.assign(c->L, 1);   // past the warm-up every layer is updated in every step
  for (auto& g : c->graph_cache)
    if (g.key == key) {
      LP_HIP(c, hipGraphLaunch(g.exec, sC));
      c->graph_replayed += 1;
      return LP_OK;
    }
  if (c->graph_cache.size() >= kMaxGraphs) {   // a caller that never repeats its buffers: stay eager
    c->graph_eager += 1;
    return enqueue_step(c, X0, target, loss_dev, sC, sW, sU, multi, updated);
  }
  LP_HIP(c, hipStreamBeginCapture(sC, hipStreamCaptureModeThreadLocal));
  const int r = enqueue_step(c, X0, target, loss_dev, sC, sW, sU, multi, updated);
  hipGraph_t graph = nullptr;
  const hipError_t e = hipStreamEndCapture(sC, &graph);
  if (r != LP_OK) {
    if (graph) (void)hipGraphDestroy(graph);
    return r;
  }
  if (e != hipSuccess) return fail_hip(c, e, "hipStreamEndCapture");
  hipGraphExec_t exec = nullptr;
  const hipError_t ei = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
  if (ei != hipSuccess) {
    (void)hipGraphDestroy(graph);
    return fail_hip(c, ei, "hipGraphInstantiate");
  }
  c->graph_cache.push_back({key, graph, exec});
  c->graph_captured += 1;
  LP_HIP(c, hipGraphLaunch(exec, sC));
  return LP_OK;
}

}  // namespace

extern "C" {

// Largest operand of a layer's products in bytes, for the kernels' 32-bit byte offsets.
constexpr unsigned long long kMaxOperandBytes = 0x7fffffffull;

int lp_create(const lp_layer_desc* layers, int L, int batch, int dtype, int loss, float lr, lp_ctx** out) {
  return guarded(nullptr, "lp_create", [&]() -> int {
    if (!layers || !out) return fail(nullptr, LP_ERR_NULL, "lp_create: layers/out is NULL");
    if (L < 1) return fail(nullptr, LP_ERR_SHAPE, "lp_create: L = %d", L);
    if (batch < 1) return fail(nullptr, LP_ERR_SHAPE, "lp_create: batch = %d", batch);
    if (dtype != LP_F32 && dtype != LP_BF16) return fail(nullptr, LP_ERR_DTYPE, "lp_create: unknown dtype %d", dtype);
    if (loss != LP_LOSS_SOFTMAX_CE && loss != LP_LOSS_MSE) return fail(nullptr, LP_ERR_DTYPE, "lp_create: unknown loss %d", loss);
    std::unique_ptr<lp_ctx> c(new lp_ctx);
    c->L = L; c->batch = batch; c->dtype = dtype; c->loss = loss; c->lr = lr;
    c->layers.resize(L);
    int prev_out_feat = -1, prevH = 0, prevW = 0, prevC = 0;
    bool prev_conv = false;
    for (int i = 0; i < L; ++i) {
      Layer& ly = c->layers[i];
      ly.d = layers[i];
      const lp_layer_desc& d = ly.d;
      auto bad = [&](int code, const char* msg) { return fail(nullptr, code, "lp_create: layer %d: %s", i + 1, msg); };
      if (d.kind != LP_LINEAR && d.kind != LP_CONV3X3) return bad(LP_ERR_DTYPE, "unknown kind");
      if (d.act < LP_ACT_IDENTITY || d.act > LP_ACT_SIGMOID) return bad(LP_ERR_DTYPE, "unknown activation");
      if (d.kind == LP_CONV3X3 && d.pool == 2 && (d.act == LP_ACT_TANH || d.act == LP_ACT_SIGMOID))
        return bad(LP_ERR_DTYPE, "a pooled convolution takes identity, ReLU or GELU");
      if (d.in < 1 || d.out < 1) return bad(LP_ERR_SHAPE, "in/out must be positive");
      if (d.delay < 0) return bad(LP_ERR_DELAY, "negative delay");
      if (i == L - 1 && d.act != LP_ACT_IDENTITY) return bad(LP_ERR_DTYPE, "the last layer must have identity activation");
      // Everything a task launcher would refuse is refused here, so that lp_step cannot fail on a shape
      // after its first launch: the kernels address their operands with 32-bit byte offsets.
      const unsigned long long es = dtype == LP_BF16 ? 2 : 4;
      if (d.kind == LP_LINEAR) {
        if (d.pool != 0 || d.H != 0 || d.W != 0) return bad(LP_ERR_SHAPE, "H, W, pool must be 0 for a linear layer");
        const unsigned long long b = (unsigned long long)batch, in = (unsigned long long)d.in, o = (unsigned long long)d.out;
        if (dtype == LP_BF16 && (b * in * es >= kMaxOperandBytes || b * o * es >= kMaxOperandBytes || in * o * es >= kMaxOperandBytes))
          return bad(LP_ERR_SHAPE, "an operand of this layer's products reaches 2 GiB (the kernels use 32-bit byte offsets)");
        if (dtype == LP_F32 && (batch > 65535 * 32 || d.in > 65535 * 32))
          return bad(LP_ERR_SHAPE, "more than 2097120 rows in an F32 product");
        ly.in_feat = d.in; ly.out_feat = d.out;
        ly.n_params = (size_t)d.in * d.out;
        ly.in_elems = (size_t)batch * d.in;
        ly.z_elems = ly.a_elems = (size_t)batch * d.out;
        if (i > 0 && prev_out_feat != d.in) return bad(LP_ERR_LAYER, "input width differs from the previous layer's output");
        prev_conv = false;
      } else {
        if (dtype != LP_BF16) return bad(LP_ERR_DTYPE, "convolution layers need an LP_BF16 context");
        if (d.H < 1 || d.W < 1) return bad(LP_ERR_SHAPE, "conv needs H, W >= 1");
        if (d.H >= 32768 || d.W >= 32768) return bad(LP_ERR_SHAPE, "conv needs H, W < 32768");
        if ((unsigned long long)batch * d.H * d.W * (d.in > d.out ? d.in : d.out) * es >= kMaxOperandBytes)
          return bad(LP_ERR_SHAPE, "an image tensor of this layer reaches 2 GiB (the kernels use 32-bit byte offsets)");
        if (i > 0 && d.out % 8 != 0) return bad(LP_ERR_SHAPE, "a conv layer other than the first needs out % 8 == 0 (dX reads 16-byte chunks)");
        if (d.pool != 0 && d.pool != 2) return bad(LP_ERR_SHAPE, "pool must be 0 or 2");
        if (d.pool == 2 && (d.H % 2 || d.W % 2)) return bad(LP_ERR_SHAPE, "pool needs even H and W");
        if (i == L - 1 && d.pool) return bad(LP_ERR_SHAPE, "the last layer cannot pool");
        if (i > 0) {
          if (!prev_conv) return bad(LP_ERR_LAYER, "a conv layer cannot follow a linear layer");
          if (prevH != d.H || prevW != d.W || prevC != d.in) return bad(LP_ERR_LAYER, "conv input shape differs from the previous layer's output");
        }
        const int p = d.pool == 2 ? 2 : 1;
        ly.in_feat = d.H * d.W * d.in;
        ly.out_feat = (d.H / p) * (d.W / p) * d.out;
        ly.n_params = (size_t)9 * d.in * d.out;
        ly.in_elems = (size_t)batch * ly.in_feat;
        ly.z_elems = (size_t)batch * d.H * d.W * d.out;
        ly.a_elems = (size_t)batch * ly.out_feat;
        prev_conv = true; prevH = d.H / p; prevW = d.W / p; prevC = d.out;
      }
      prev_out_feat = ly.out_feat;
      ly.delay = d.delay;
      ly.ring_slots = d.delay + 1;
    }
    layout_workspace(c.get());
    *out = c.release();
    return LP_OK;
  });
}

int lp_destroy(lp_ctx* c) {
  return guarded(nullptr, "lp_destroy", [&]() -> int {
    if (!c) return LP_ERR_NULL;
    if (c->events_ready) {
      for (auto* v : {&c->ev_dy, &c->ev_dx, &c->ev_dw, &c->ev_split, &c->ev_upd})
        for (hipEvent_t e : *v)
          if (e) (void)hipEventDestroy(e);
      for (hipEvent_t e : {c->ev_fork, c->ev_join_w, c->ev_join_u, c->ev_loss[0], c->ev_loss[1], c->ev_bdone[0], c->ev_bdone[1]})
        if (e) (void)hipEventDestroy(e);
    }
    drop_graphs(c);
    for (auto& r : c->prof_recs) { (void)hipEventDestroy(r.e0); (void)hipEventDestroy(r.e1); }
    for (hipEvent_t e : c->prof_free) (void)hipEventDestroy(e);
    delete c;
    return LP_OK;
  });
}

const char* lp_last_error(const lp_ctx* c) { return c ? c->err.c_str() : g_create_error.c_str(); }

int lp_workspace_bytes(const lp_ctx* c, size_t* bytes) {
  if (!c || !bytes) return LP_ERR_NULL;
  *bytes = c->ws_bytes;
  return LP_OK;
}

int lp_bind_workspace(lp_ctx* c, void* dev_ptr, size_t bytes) {
  return guarded(c, "lp_bind_workspace", [&]() -> int {
    if (!c) return LP_ERR_NULL;
    if (!dev_ptr) return fail(c, LP_ERR_NULL, "lp_bind_workspace: dev_ptr is NULL");
    if ((uintptr_t)dev_ptr % kAlign) return fail(c, LP_ERR_WORKSPACE, "lp_bind_workspace: pointer not %zu-byte aligned", kAlign);
    if (bytes < c->ws_bytes) return fail(c, LP_ERR_WORKSPACE, "lp_bind_workspace: %zu bytes given, %zu needed", bytes, c->ws_bytes);
    drop_graphs(c);
    c->ws = (char*)dev_ptr;
    c->n = 0;
    for (Layer& ly : c->layers) { ly.weights_set = false; ly.cur = 0; }
    return LP_OK;
  });
}

int lp_set_weights(lp_ctx* c, int l, const float* W, int is_device, void* stream) {
  return guarded(c, "lp_set_weights", [&]() -> int {
    if (!c) return LP_ERR_NULL;
    if (int r = check_layer(c, l)) return r;
    if (!W) return fail(c, LP_ERR_NULL, "lp_set_weights: W is NULL");
    if (int r = need_ws(c)) return r;
    Layer& ly = c->layers[l - 1];
    hipStream_t s = (hipStream_t)stream;
    note_stream(c, s);
    float* master = (float*)(c->ws + ly.off_master);
    if (is_device) LP_HIP(c, hipMemcpyAsync(master, W, ly.n_params * 4, hipMemcpyDeviceToDevice, s));
    else {
      LP_HIP(c, hipStreamSynchronize(s));
      LP_HIP(c, hipMemcpy(master, W, ly.n_params * 4, hipMemcpyHostToDevice));
    }
    if (ly.retimed) {
      // every held version: the steps to come read these weights until versions written after this call come of age
      for (int v = 0; v < ly.n_versions; ++v) LP_HIP(c, lp::launch_cast_bf16(master, version_slot(c, ly, v), ly.n_params, s));
    } else if (is_bf16(c)) {
      LP_HIP(c, lp::launch_cast_bf16(master, c->ws + ly.off_work[ly.cur], ly.n_params, s));
    }
    // the table the F epilogue of a GELU layer looks its activation up in: made ready here, outside any step
    if (is_bf16(c) && ly.d.kind == LP_LINEAR && ly.d.act == LP_ACT_GELU && !c->gelu_lut) LP_HIP(c, lp::gelu_lut_bf16(&c->gelu_lut, s));
    if (is_bf16(c) && ly.d.act == LP_ACT_GELU && !c->gelu_grad_lut) LP_HIP(c, lp::gelu_grad_lut_f32(&c->gelu_grad_lut, s));
    ly.weights_set = true;
    return LP_OK;
  });
}

int lp_get_weights(lp_ctx* c, int l, float* dst, int is_device, void* stream) {
  return guarded(c, "lp_get_weights", [&]() -> int {
    if (!c) return LP_ERR_NULL;
    if (int r = check_layer(c, l)) return r;
    if (!dst) return fail(c, LP_ERR_NULL, "lp_get_weights: dst is NULL");
    if (int r = need_weights(c, l)) return r;
    Layer& ly = c->layers[l - 1];
    hipStream_t s = (hipStream_t)stream;
    const float* master = (const float*)(c->ws + ly.off_master);
    if (is_device) LP_HIP(c, hipMemcpyAsync(dst, master, ly.n_params * 4, hipMemcpyDeviceToDevice, s));
    else {
      // run-ahead steps do not join the update stream into any other: wait for all of them
      if (c->run_ahead) for (hipStream_t t : c->streams_seen) LP_HIP(c, hipStreamSynchronize(t));
      LP_HIP(c, hipStreamSynchronize(s));
      LP_HIP(c, hipMemcpy(dst, master, ly.n_params * 4, hipMemcpyDeviceToHost));
    }
    return LP_OK;
  });
}

int lp_cast(lp_ctx* c, const float* src, void* dst, size_t n, void* stream) {
  return guarded(c, "lp_cast", [&]() -> int {
    if (!c) return LP_ERR_NULL;
    if (!src || !dst) return fail(c, LP_ERR_NULL, "lp_cast: src/dst is NULL");
    if ((uintptr_t)src % 16 || (uintptr_t)dst % 16) return fail(c, LP_ERR_SHAPE, "lp_cast: src and dst must be 16-byte aligned");
    if (n == 0) return LP_OK;
    note_stream(c, (hipStream_t)stream);
    if (is_bf16(c)) LP_HIP(c, lp::launch_cast_bf16(src, dst, n, (hipStream_t)stream));
    else LP_HIP(c, hipMemcpyAsync(dst, src, n * 4, hipMemcpyDeviceToDevice, (hipStream_t)stream));
    return LP_OK;
  });
}

int lp_forward(lp_ctx* c, int l, const void* X, void* Z, void* A, void* stream) {
  return guarded(c, "lp_forward", [&]() -> int {
    if (!c) return LP_ERR_NULL;
    if (int r = check_layer(c, l)) return r;
    if (!X) return fail(c, LP_ERR_NULL, "lp_forward: X is NULL");
    if (!Z && !A) return fail(c, LP_ERR_NULL, "lp_forward: both outputs are NULL");
    Layer& ly = c->layers[l - 1];
    if (ly.d.kind == LP_CONV3X3 && ly.d.pool == 2 && !Z) return fail(c, LP_ERR_NULL, "lp_forward: a pooled layer needs Z");
    if (int r = need_weights(c, l)) return r;
    note_stream(c, (hipStream_t)stream);
    LP_HIP(c, do_forward(c, ly, X, Z, A, (hipStream_t)stream));
    return LP_OK;
  });
}

int lp_loss_grad(lp_ctx* c, const void* ZL, const void* target, void* dYL, float* loss_dev, void* stream) {
  return guarded(c, "lp_loss_grad", [&]() -> int {
    if (!c) return LP_ERR_NULL;
    if (!ZL || !target || !dYL) return fail(c, LP_ERR_NULL, "lp_loss_grad: ZL/target/dYL is NULL");
    if (int r = need_ws(c)) return r;
    note_stream(c, (hipStream_t)stream);
    LP_HIP(c, do_loss(c, ZL, target, dYL, loss_dev, (hipStream_t)stream));
    return LP_OK;
  });
}

int lp_loss_grad_static(lp_ctx* c, const void* ZL, const void* target, void* dYL, float* loss_dev, void* stream) {
  return guarded(c, "lp_loss_grad_static", [&]() -> int {
    if (!c) return LP_ERR_NULL;
    if (!ZL || !target || !dYL) return fail(c, LP_ERR_NULL, "lp_loss_grad_static: ZL/target/dYL is NULL");
    const Layer& last = c->layers[c->L - 1];
    const bool mse = c->loss == LP_LOSS_MSE;
    const size_t need = lp::loss_partials_count(mse, c->batch, last.out_feat), have = lp::static_loss_partials_capacity();
    if (need > have)
      return fail(c, LP_ERR_SHAPE, "lp_loss_grad_static: %zu partial sums needed, the static scratch holds %zu (%s); use lp_loss_grad with a workspace",
                  need, have, mse ? "batch x D_L <= 536870912 elements" : "batch <= 65536 rows");
    float* partials = nullptr;
    LP_HIP(c, lp::static_loss_partials(&partials));
    hipStream_t s = (hipStream_t)stream;
    if (mse) LP_HIP(c, lp::launch_mse(is_bf16(c), ZL, target, dYL, loss_dev, partials, c->batch, last.out_feat, s));
    else LP_HIP(c, lp::launch_softmax_ce(is_bf16(c), ZL, (const int*)target, dYL, loss_dev, partials, c->batch, last.out_feat, s));
    return LP_OK;
  });
}

int lp_act_grad(lp_ctx* c, int l, const void* dA, const void* S, void* dY, void* stream) {
  return guarded(c, "lp_act_grad", [&]() -> int {
    if (!c) return LP_ERR_NULL;
    if (int r = check_layer(c, l)) return r;
    Layer& ly = c->layers[l - 1];
    if (!dA || !dY || (!S && ly.d.act != LP_ACT_IDENTITY)) return fail(c, LP_ERR_NULL, "lp_act_grad: dA/S/dY is NULL");
    if (ly.d.kind == LP_CONV3X3 && ly.d.pool == 2) {
      if (!S) return fail(c, LP_ERR_NULL, "lp_act_grad: a pooled layer needs S = Z");
      if (dA == dY) return fail(c, LP_ERR_SHAPE, "lp_act_grad: dY may not alias dA on a pooled layer");
    }
    note_stream(c, (hipStream_t)stream);
    LP_HIP(c, do_act_grad(c, ly, dA, S, dY, (hipStream_t)stream));
    return LP_OK;
  });
}

int lp_grad_act(lp_ctx* c, int l, const void* dY, void* dX, int col0, int col1, void* stream) {
  return guarded(c, "lp_grad_act", [&]() -> int {
    if (!c) return LP_ERR_NULL;
    if (int r = check_layer(c, l)) return r;
    if (!dY || !dX) return fail(c, LP_ERR_NULL, "lp_grad_act: dY/dX is NULL");
    Layer& ly = c->layers[l - 1];
    if (col0 < 0 || col1 > ly.d.in || col0 >= col1) return fail(c, LP_ERR_SHAPE, "lp_grad_act: column range [%d,%d) outside [0,%d)", col0, col1, ly.d.in);
    if (int r = need_weights(c, l)) return r;
    note_stream(c, (hipStream_t)stream);
    LP_HIP(c, do_grad_act(c, ly, dY, dX, col0, col1, (hipStream_t)stream));
    return LP_OK;
  });
}

int lp_grad_weight(lp_ctx* c, int l, const void* X, const void* dY, float* G, void* stream) {
  return guarded(c, "lp_grad_weight", [&]() -> int {
    if (!c) return LP_ERR_NULL;
    if (int r = check_layer(c, l)) return r;
    if (!X || !dY) return fail(c, LP_ERR_NULL, "lp_grad_weight: X/dY is NULL");
    if (int r = need_ws(c)) return r;
    Layer& ly = c->layers[l - 1];
    note_stream(c, (hipStream_t)stream);
    if (!G) {
      LP_HIP(c, enqueue_G(c, ly, X, dY, c->n + 1, (hipStream_t)stream));
      return LP_OK;
    }
    LP_HIP(c, do_grad_weight(c, ly, X, dY, G, (hipStream_t)stream));
    return LP_OK;
  });
}

int lp_update(lp_ctx* c, int l, const float* G, void* stream) {
  return guarded(c, "lp_update", [&]() -> int {
    if (!c) return LP_ERR_NULL;
    if (int r = check_layer(c, l)) return r;
    if (int r = need_weights(c, l)) return r;
    Layer& ly = c->layers[l - 1];
    if (ly.retimed) return fail(c, LP_ERR_STATE, "lp_update: layer %d has the retimed update; its G task inside lp_step applies the gradient", l);
    if (!G) {
      const long src = c->n + 1 - ly.delay;
      if (src < 1) return LP_OK;  // the delay elements are still empty
      note_stream(c, (hipStream_t)stream);
      LP_HIP(c, enqueue_update(c, ly, src, (hipStream_t)stream));
      if (is_bf16(c)) ly.cur ^= 1;
      return LP_OK;
    }
    note_stream(c, (hipStream_t)stream);
    LP_HIP(c, do_update(c, ly, G, (hipStream_t)stream));
    if (is_bf16(c)) ly.cur ^= 1;
    return LP_OK;
  });
}

int lp_set_delta_split(lp_ctx* c, int l, int cols) {
  return guarded(c, "lp_set_delta_split", [&]() -> int {
    if (!c) return LP_ERR_NULL;
    if (int r = check_layer(c, l)) return r;
    Layer& ly = c->layers[l - 1];
    if (l == 1 && cols != 0) return fail(c, LP_ERR_LAYER, "lp_set_delta_split: layer 1 has no delta task");
    if (cols < 0 || cols >= ly.d.in) return fail(c, LP_ERR_SHAPE, "lp_set_delta_split: %d columns outside [0, %d)", cols, ly.d.in);
    ly.split_cols = cols;
    return LP_OK;
  });
}

int lp_set_factor_ring(lp_ctx* c, int l, int enable) {
  return guarded(c, "lp_set_factor_ring", [&]() -> int {
    if (!c) return LP_ERR_NULL;
    if (c->ws) return fail(c, LP_ERR_STATE, "lp_set_factor_ring: call it before lp_bind_workspace (it changes the workspace size)");
    if (!is_bf16(c)) return fail(c, LP_ERR_DTYPE, "lp_set_factor_ring: needs an LP_BF16 context");
    if (l != 0)
      if (int r = check_layer(c, l)) return r;
    if (l != 0 && c->layers[l - 1].d.kind != LP_LINEAR) return fail(c, LP_ERR_LAYER, "lp_set_factor_ring: layer %d is not a linear layer", l);
    // A layer whose stand-alone G product is not the plain tiled GEMM that the fused update runs -- K cut into ranges
    // (few output tiles, long batch), or the short-vector kernels of a layer with a handful of outputs -- is summed
    // in another order there: such a layer keeps its product ring.
    auto k_is_cut = [&](const Layer& ly) {
      return lp::gemm_bf16_splitk_splits(ly.d.in, ly.d.out, c->batch) > 1 || lp::gemm_skinny_shape(c->batch, ly.d.in, ly.d.out);
    };
    if (l != 0 && enable && c->layers[l - 1].retimed)
      return fail(c, LP_ERR_LAYER, "lp_set_factor_ring: layer %d has the retimed update, which keeps no gradients", l);
    if (l != 0 && enable && k_is_cut(c->layers[l - 1]))
      return fail(c, LP_ERR_LAYER, "lp_set_factor_ring: the G product of layer %d is split over K (or runs on the few-outputs kernels) at this batch size; it keeps the product ring", l);
    for (int i = 0; i < c->L; ++i) {
      Layer& ly = c->layers[i];
      if ((l == 0 || i == l - 1) && ly.d.kind == LP_LINEAR) ly.factor_ring = enable != 0 && !k_is_cut(ly) && !ly.retimed;
    }
    layout_workspace(c);
    return LP_OK;
  });
}

int lp_set_retimed_update(lp_ctx* c, int l, int enable) {
  return guarded(c, "lp_set_retimed_update", [&]() -> int {
    if (!c) return LP_ERR_NULL;
    if (c->ws) return fail(c, LP_ERR_STATE, "lp_set_retimed_update: call it before lp_bind_workspace (it changes the workspace size)");
    if (!is_bf16(c)) return fail(c, LP_ERR_DTYPE, "lp_set_retimed_update: needs an LP_BF16 context");
    if (l != 0)
      if (int r = check_layer(c, l)) return r;
    // The update rides in the kernel that finishes G, in the summation order of lp_grad_weight: for a linear layer the
    // epilogue of the tiled GEMM or of the few-outputs kernel, or the kernel that adds the partial sums where K is cut into
    // ranges; for a convolution the kernel that adds the split-K partial sums.  A convolution whose G product is not split
    // has no such kernel, and keeps its gradient ring.
    auto eligible = [&](const Layer& ly) {
      if (ly.d.kind == LP_CONV3X3) return lp::conv_grad_weight_scratch_bytes(conv_desc(c, ly)) > 0;
      return !ly.factor_ring;
    };
    if (l != 0 && enable && !eligible(c->layers[l - 1]))
      return fail(c, LP_ERR_LAYER, "lp_set_retimed_update: layer %d has a factor ring, or is a convolution whose G product is not split over K at "
                  "this batch size; it keeps its gradient ring", l);
    for (int i = 0; i < c->L; ++i) {
      Layer& ly = c->layers[i];
      if (l == 0 || i == l - 1) ly.retimed = enable != 0 && eligible(ly);
    }
    layout_workspace(c);
    return LP_OK;
  });
}

int lp_set_graphs(lp_ctx* c, int enable) {
  return guarded(c, "lp_set_graphs", [&]() -> int {
    if (!c) return LP_ERR_NULL;
    if (c->ws) return fail(c, LP_ERR_STATE, "lp_set_graphs: call it before lp_bind_workspace (it changes the workspace size)");
    if (enable && c->run_ahead) return fail(c, LP_ERR_STATE, "lp_set_graphs: not together with forward run-ahead");
    c->graphs = enable != 0;
    layout_workspace(c);
    return LP_OK;
  });
}

int lp_graph_stats(const lp_ctx* c, long* captured, long* replayed, long* eager) {
  if (!c) return LP_ERR_NULL;
  if (captured) *captured = c->graph_captured;
  if (replayed) *replayed = c->graph_replayed;
  if (eager) *eager = c->graph_eager;
  return LP_OK;
}

int lp_set_run_ahead(lp_ctx* c, int enable) {
  return guarded(c, "lp_set_run_ahead", [&]() -> int {
    if (!c) return LP_ERR_NULL;
    if (c->ws) return fail(c, LP_ERR_STATE, "lp_set_run_ahead: call it before lp_bind_workspace (it changes the workspace size)");
    if (enable && !is_bf16(c)) return fail(c, LP_ERR_DTYPE, "lp_set_run_ahead: needs an LP_BF16 context (F32 updates the weights in place)");
    if (enable && c->graphs) return fail(c, LP_ERR_STATE, "lp_set_run_ahead: not together with graph replay");
    c->run_ahead = enable != 0;
    layout_workspace(c);
    return LP_OK;
  });
}

int lp_set_fused_hadamard(lp_ctx* c, int enable) {
  return guarded(c, "lp_set_fused_hadamard", [&]() -> int {
    if (!c) return LP_ERR_NULL;
    if ((enable != 0) != c->fuse_hadamard) drop_graphs(c);   // captured steps hold the other kernel sequence
    c->fuse_hadamard = enable != 0;
    return LP_OK;
  });
}

int lp_advance(lp_ctx* c) {
  if (!c) return LP_ERR_NULL;
  c->n += 1;
  return LP_OK;
}

int lp_step(lp_ctx* c, const void* X0, const void* target, const int* delay, float* loss_dev, void* const* streams, int n_streams) {
  return guarded(c, "lp_step", [&]() -> int {
    if (!c) return LP_ERR_NULL;
    if (!X0 || !target) return fail(c, LP_ERR_NULL, "lp_step: X0/target is NULL");
    if (!streams || n_streams < 1) return fail(c, LP_ERR_NULL, "lp_step: needs at least one stream");
    if (int r = need_ws(c)) return r;
    for (int l = 1; l <= c->L; ++l)
      if (int r = need_weights(c, l)) return r;
    if (delay) {
      for (int l = 0; l < c->L; ++l)
        if (delay[l] < 0 || delay[l] > c->layers[l].d.delay)
          return fail(c, LP_ERR_DELAY, "lp_step: delay[%d] = %d outside [0, %d]", l, delay[l], c->layers[l].d.delay);
      for (int l = 0; l < c->L; ++l)
        if (c->layers[l].retimed && delay[l] != c->layers[l].d.delay)
          return fail(c, LP_ERR_DELAY, "lp_step: layer %d has the retimed update, whose delay is fixed at %d (delay[%d] = %d)", l + 1, c->layers[l].d.delay, l, delay[l]);
      for (int l = 0; l < c->L; ++l) c->layers[l].delay = delay[l];
    }
    if (c->run_ahead) {
      if (n_streams < 4) return fail(c, LP_ERR_STATE, "lp_step: forward run-ahead needs 4 stream handles, %d given", n_streams);
      if (streams[3] == streams[0]) return fail(c, LP_ERR_STATE, "lp_step: forward run-ahead needs a forward stream (streams[3]) other than streams[0]");
      return step_run_ahead(c, X0, target, loss_dev, streams);
    }
    const bool multi = n_streams > 1;
    hipStream_t sC = (hipStream_t)streams[0];
    hipStream_t sW = multi ? (hipStream_t)streams[1] : sC;
    hipStream_t sU = multi ? (hipStream_t)streams[2 % n_streams] : sC;
    note_stream(c, sC); note_stream(c, sW); note_stream(c, sU);
    if (multi)
      if (int r = ensure_events(c)) return r;

    const int L = c->L;
    const long n = c->n + 1;
    const bool bf = is_bf16(c);
    std::vector<char> updated;
    if (int r = run_or_replay_step(c, X0, target, loss_dev, sC, sW, sU, multi, updated)) return r;
    if (bf)
      for (int i = 0; i < L; ++i)
        if (updated[i] && !c->layers[i].retimed) c->layers[i].cur ^= 1;
    c->n = n;
    return LP_OK;
  });
}

int lp_step_index(const lp_ctx* c, long* n) {
  if (!c || !n) return LP_ERR_NULL;
  *n = c->n;
  return LP_OK;
}

int lp_sync(lp_ctx* c) {
  return guarded(c, "lp_sync", [&]() -> int {
    if (!c) return LP_ERR_NULL;
    for (hipStream_t s : c->streams_seen) LP_HIP(c, hipStreamSynchronize(s));
    return LP_OK;
  });
}

int lp_tensor(lp_ctx* c, int l, int which, void** dev_ptr, size_t* bytes) {
  return guarded(c, "lp_tensor", [&]() -> int {
    if (!c) return LP_ERR_NULL;
    if (!dev_ptr || !bytes) return fail(c, LP_ERR_NULL, "lp_tensor: dev_ptr/bytes is NULL");
    if (int r = check_layer(c, l)) return r;
    if (int r = need_ws(c)) return r;
    Layer& ly = c->layers[l - 1];
    const size_t es = esize(c);
    *dev_ptr = nullptr; *bytes = 0;
    switch (which) {
      case LP_T_MASTER_W: *dev_ptr = c->ws + ly.off_master; *bytes = ly.n_params * 4; break;
      case LP_T_WORK_W: *dev_ptr = work_w(c, ly); *bytes = ly.n_params * es; break;
      case LP_T_A: if (ly.has_A) { *dev_ptr = c->ws + ly.off_A[c->n & 1]; *bytes = ly.a_elems * es; } break;
      case LP_T_Z: if (ly.has_Z) { *dev_ptr = c->ws + ly.off_Z[c->n & 1]; *bytes = ly.z_elems * es; } break;
      case LP_T_DA:   // not materialised when the layer above applies the Hadamard product in its dX epilogue
        if (ly.has_dA && !(l < c->L && hadamard_fused(c, c->layers[l], ly))) { *dev_ptr = c->ws + ly.off_dA; *bytes = ly.a_elems * es; }
        break;
      case LP_T_DY: *dev_ptr = c->ws + ly.off_dY; *bytes = ly.z_elems * es; break;
      case LP_T_G_LAST: if (c->n >= 1 && !ly.factor_ring && !ly.retimed) { *dev_ptr = ring_slot(c, ly, c->n); *bytes = ly.n_params * 4; } break;
      default: return fail(c, LP_ERR_DTYPE, "lp_tensor: unknown tensor id %d", which);
    }
    return LP_OK;
  });
}

int lp_probe_mfma(float* out_dev, size_t out_elems, int workgroups, int iters, int uniform_values, void* stream) {
  if (!out_dev) return LP_ERR_NULL;
  if (workgroups < 1 || iters < 0 || out_elems < (size_t)workgroups * 512) return LP_ERR_SHAPE;
  return lp::launch_mfma_only(out_dev, workgroups, iters, uniform_values != 0, (hipStream_t)stream) == hipSuccess ? LP_OK : LP_ERR_HIP;
}

int lp_profile(lp_ctx* c, int enable) {
  if (!c) return LP_ERR_NULL;
  c->prof_on = enable != 0;
  return LP_OK;
}

namespace {
int profile_collect(lp_ctx* c) {
  if (c->prof_ms.empty()) {
    c->prof_ms.assign((size_t)LP_TASK_COUNT * (c->L + 1), 0.0);
    c->prof_n.assign((size_t)LP_TASK_COUNT * (c->L + 1), 0);
  }
  for (auto& r : c->prof_recs) {
    LP_HIP(c, hipEventSynchronize(r.e1));
    float ms = 0.f;
    LP_HIP(c, hipEventElapsedTime(&ms, r.e0, r.e1));
    const size_t k = (size_t)r.task * (c->L + 1) + r.layer;
    c->prof_ms[k] += ms;
    c->prof_n[k] += 1;
    c->prof_free.push_back(r.e0);
    c->prof_free.push_back(r.e1);
  }
  c->prof_recs.clear();
  return LP_OK;
}
}  // namespace

int lp_profile_read(lp_ctx* c, int task, double* total_ms, long* launches, int reset) {
  return guarded(c, "lp_profile_read", [&]() -> int {
    if (!c) return LP_ERR_NULL;
    if (task < 0 || task >= LP_TASK_COUNT) return fail(c, LP_ERR_DTYPE, "lp_profile_read: unknown task %d", task);
    if (int r = profile_collect(c)) return r;
    double ms = 0.0;
    long n = 0;
    for (int l = 0; l <= c->L; ++l) {
      const size_t k = (size_t)task * (c->L + 1) + l;
      ms += c->prof_ms[k];
      n += c->prof_n[k];
      if (reset) { c->prof_ms[k] = 0; c->prof_n[k] = 0; }
    }
    if (total_ms) *total_ms = ms;
    if (launches) *launches = n;
    return LP_OK;
  });
}

int lp_profile_read_layer(lp_ctx* c, int task, int l, double* total_ms, long* launches, int reset) {
  return guarded(c, "lp_profile_read_layer", [&]() -> int {
    if (!c) return LP_ERR_NULL;
    if (task < 0 || task >= LP_TASK_COUNT) return fail(c, LP_ERR_DTYPE, "lp_profile_read_layer: unknown task %d", task);
    if (int r = check_layer(c, l)) return r;
    if (int r = profile_collect(c)) return r;
    const size_t k = (size_t)task * (c->L + 1) + l;
    if (total_ms) *total_ms = c->prof_ms[k];
    if (launches) *launches = c->prof_n[k];
    if (reset) { c->prof_ms[k] = 0; c->prof_n[k] = 0; }
    return LP_OK;
  });
}

}  // extern "C"
