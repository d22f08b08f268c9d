// Host side of the SpecPipe stage library: argument checks against a host mirror of
// the tree, workspace carving, the page allocator of the paged cache, and the per-layer
// launch sequence (replayed from a HIP graph for shapes seen before).  No device memory
// is allocated here and nothing waits for the GPU except sp_tree_read and
// sp_profile_end.
#include <cmath>
#include <cstring>
#include <new>
#include <vector>

#include "../../include/specpipe.h"
#include "sp_launch.h"

static_assert(SP_T == SP_MAX_TREE_NODES, "tree capacity");
static_assert(SP_W == SP_ANC_WORDS, "mask words");
static_assert(SP_BATCH == SP_MAX_BATCH_REQ, "batch capacity");
static_assert(SP_SAMPLE_MAX_K == SP_MAX_SAMPLE_TOP_K, "candidates of a stochastic verification");

namespace {

struct HostReq {
  bool active = false;
  long long base = 0;
  int cap = 0, P = 0, T = 0;
  short parent[SP_T];
  unsigned char fwd[SP_T];      // node's K/V rows exist at this stage
  bool pending = false;         // a prune awaits its cache compaction
  int pend_mode = 0, pend_node = 0;
  short pend_tab_new[SP_T];     // old node -> new index, -1 gone
  std::vector<int> pages;       // paged cache: physical page of every logical page the request holds
  // A prune decided on the device (sp_tree_prune_verified) whose outcome the mirror has not taken yet:
  // the verified node arrives in pinned host memory, entry unrec_slot, once the stage's copy event is done.
  bool unrec = false;
  int unrec_slot = 0;
};

inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

struct Workspace {
  RowInfo* rows = nullptr;
  float* cs = nullptr;
  float* h = nullptr;
  void* xn = nullptr;
  void* qbuf = nullptr;
  void* attn = nullptr;
  void* act = nullptr;
  float* part = nullptr;
  float* attn_part = nullptr;
  AttnPlan* plan = nullptr;            // device copy of the current call's plan
  size_t part_floats = 0;
  size_t attn_units = 0;
  size_t total = 0;
};

inline int elt_bytes(int dtype) { return dtype == SP_BF16 ? 2 : 4; }

// Lays the workspace out from `base` (may be null: sizes only).
Workspace carve(const sp_config& c, char* base) {
  Workspace w;
  const size_t MB = align_up((size_t)c.max_batch_nodes, 16);
  const size_t eb = elt_bytes(c.dtype);
  const size_t dq = (size_t)c.n_q_heads * c.d_head, dkv = (size_t)c.n_kv_heads * c.d_head;
  const size_t nqkv = dq + 2 * dkv;
  size_t off = 0;
  auto take = [&](size_t bytes) { char* p = base ? base + off : nullptr; off += align_up(bytes); return (void*)p; };
  w.rows = (RowInfo*)take(MB * sizeof(RowInfo));
  w.cs = (float*)take(MB * c.d_head * sizeof(float));
  w.h = (float*)take(MB * c.d_model * sizeof(float));
  w.xn = take(MB * c.d_model * eb);
  w.qbuf = take(MB * dq * eb);
  w.attn = take(MB * dq * eb);
  w.act = take(MB * (size_t)c.d_ff * eb);
  // partial sums of the split projections, or the unfused gate/up output
  const size_t part_rows = MB > 1024 ? MB : 1024;
  const size_t nmax = nqkv > (size_t)c.d_model ? nqkv : (size_t)c.d_model;
  size_t pf = part_rows * nmax;
  const size_t gu = MB * 2 * (size_t)c.d_ff;
  if (gu > pf) pf = gu;
  w.part_floats = pf;
  w.part = (float*)take(pf * sizeof(float));
  // split-KV attention partials: (max, sum, d_head outputs) per (row, head, chunk)
  w.attn_units = (MB > 64 ? MB : 64) * (size_t)c.n_q_heads * 32;
  w.attn_part = (float*)take(w.attn_units * (size_t)(c.d_head + 2) * sizeof(float));
  w.plan = (AttnPlan*)take(sizeof(AttnPlan));
  w.total = off;
  return w;
}

int check_config(const sp_config* c) {
  if (!c) return SP_E_INVALID;
  if (c->n_layers < 1 || c->d_model < 8 || c->n_q_heads < 1 || c->n_kv_heads < 1 || c->d_ff < 8) return SP_E_INVALID;
  if (c->n_q_heads % c->n_kv_heads) return SP_E_INVALID;
  if (c->dtype != SP_F32 && c->dtype != SP_BF16) return SP_E_INVALID;
  if (c->max_requests < 1 || c->max_tree_nodes < 1 || c->max_tree_nodes > SP_MAX_TREE_NODES) return SP_E_INVALID;
  if (c->max_batch_nodes < 1 || c->kv_slots < 1) return SP_E_INVALID;
  if (c->d_model % 8 || c->d_ff % 8) return SP_E_UNSUPPORTED;
  if (c->d_head != 64 && c->d_head != 128) return SP_E_UNSUPPORTED;
  if (!(c->rms_eps > 0.f) || !(c->rope_theta > 1.f)) return SP_E_INVALID;
  if (c->flags & SP_FLAG_PAGED_KV) {
    // a page holds whole 32-slot attention tiles
    const int pg = c->page_slots;
    if (pg < 32 || pg > 4096 || (pg & (pg - 1))) return SP_E_INVALID;
    if (c->kv_slots % pg) return SP_E_INVALID;
  }
  return SP_OK;
}

inline bool is_paged(const sp_config& c) { return (c.flags & SP_FLAG_PAGED_KV) != 0; }
inline size_t page_table_bytes(const sp_config& c) {
  if (!is_paged(c)) return 0;
  return align_up((size_t)c.max_requests * (size_t)(c.kv_slots / c.page_slots) * sizeof(int));
}

}  // namespace

// Scratch of the allocation-free entry point (sp_stage_verify_head_noalloc): a fixed array in the
// library's own device image, so that a call needs no workspace from anybody.  Every GPU the library
// runs on holds one copy at its own address; the name below is only a host-side handle, the address
// is asked for once per device (sp_stage_create) and kept in g_noalloc_scratch[device].
#define SP_NOALLOC_MAX_DEVICES 64
static __device__ __align__(256) unsigned char sp_noalloc_scratch[SP_NOALLOC_SCRATCH_BYTES];
static void* g_noalloc_scratch[SP_NOALLOC_MAX_DEVICES];

struct sp_stage {
  sp_config cfg;
  std::vector<sp_layer_weights> W;
  sp_buffers buf;
  sp_sizes sizes;
  ReqMeta* d_meta = nullptr;
  ReqTables* d_tables = nullptr;
  Workspace ws;
  KvGeom geom;
  std::vector<HostReq> reqs;
  // paged cache: the allocator lives on the host, the page tables on the device
  int n_pages = 0;
  int* d_page_table = nullptr;
  std::vector<int> free_pages;
  // Forward calls of a shape seen before replay a HIP graph of their launches (all but the first
  // and the last kernel, which carry the caller's pointers and the call's plan).
  struct FwdGraph {
    int M, qt, items, any_split, units;
    int seen;
    int S_last;                // split count of the last layer's down projection (the write-out folds it)
    bool failed;
    hipGraphExec_t exec;
  };
  std::vector<FwdGraph> graphs;
  bool use_graphs = true;
  bool fast = false;           // bf16 MFMA kernels in use
  bool packed = false;         // weights are in MFMA fragment order
  int* pin_nodes = nullptr;    // pinned host copy of the device-side verification results (sp_tree_prune_verified)
  hipEvent_t rec_ev = nullptr; // done when that copy has arrived
  int n_cu = 256;              // compute units of the device
  // The O projections of all the stage's layers together fit in half of the 256 MB Infinity Cache: they are read with
  // ordinary loads and so stay there from one step to the next, while every other weight streams past it.
  bool o_resident = false;
  int device = 0;              // the device that was current at sp_stage_create
  int last_hip = 0;
  // profiling
  int prof_kind = 0, prof_max = 0, prof_n = 0;
  // Sampling: launches of the profiled kind are counted in groups (the launches of one forward call);
  // every prof_every-th group is bracketed, the others run untouched (and may replay a graph).
  int prof_every = 1, prof_seen = 0, prof_group = 1;
  std::vector<hipEvent_t> prof_ev;
};

namespace {

inline int hip_fail(sp_stage* s, hipError_t e) {
  s->last_hip = (int)e;
  return SP_E_HIP;
}

// Brackets a launch with events when its kind is being profiled.
struct ProfScope {
  sp_stage* s;
  hipStream_t st;
  bool on;
  ProfScope(sp_stage* s_, int kind, hipStream_t st_) : s(s_), st(st_) {
    on = false;
    if (s->prof_kind == kind && s->prof_n < s->prof_max)
      on = ((s->prof_seen++ / s->prof_group) % s->prof_every) == 0;
    if (on) (void)hipEventRecord(s->prof_ev[2 * s->prof_n], st);
  }
  ~ProfScope() {
    if (on) { (void)hipEventRecord(s->prof_ev[2 * s->prof_n + 1], st); ++s->prof_n; }
  }
};

size_t tables_meta_bytes(const sp_config& c) { return align_up((size_t)c.max_requests * sizeof(ReqMeta)); }

// Paged cache: make request `req` hold the pages of its first `slots` logical slots.  Growth
// takes pages from the free list and sends their ids to the device table; shrinking returns
// pages (their table entries stay behind, unused).  Everything runs in stream order, so a page
// can be handed to another request as soon as the host has let go of it.
hipError_t pages_resize(sp_stage* s, int req, int slots, hipStream_t st) {
  HostReq& r = s->reqs[req];
  const int pg = s->cfg.page_slots;
  const int want = (slots + pg - 1) / pg;
  const int have = (int)r.pages.size();
  if (want > have) {
    for (int i = have; i < want; ++i) { r.pages.push_back(s->free_pages.back()); s->free_pages.pop_back(); }
    return sp_launch_pages_set(s->d_page_table, s->n_pages, req, have, want - have, r.pages.data() + have, st);
  }
  for (int i = have - 1; i >= want; --i) s->free_pages.push_back(r.pages[i]);
  r.pages.resize(want);
  return hipSuccess;
}
inline int pages_for(const sp_stage* s, int slots) { return (slots + s->cfg.page_slots - 1) / s->cfg.page_slots; }

void reconcile(sp_stage* s, int req);

HostReq* get_req(sp_stage* s, int req) {
  if (!s || req < 0 || req >= (int)s->reqs.size() || !s->reqs[req].active) return nullptr;
  if (s->reqs[req].unrec) reconcile(s, req);
  return &s->reqs[req];
}

// Host mirror of a prune: same result as the device kernel, computed from the
// parent list instead of the bitmask.  Fills tab_new and returns counts.
void mirror_prune(HostReq& r, int mode, int node, int* n_tab, int* n_commit) {
  bool in_col[SP_T];
  for (int i = 0; i < r.T; ++i)
    in_col[i] = mode == SP_CLEAR || (i == node) || (r.parent[i] >= 0 && in_col[r.parent[i]]);
  int commit = 0;
  if (mode == SP_ACCEPT) for (int j = node; j >= 0; j = r.parent[j]) ++commit;
  short parent_new[SP_T];
  unsigned char fwd_new[SP_T];
  int k = 0;
  for (int i = 0; i < r.T; ++i) {
    const bool keep = (mode == SP_ACCEPT) ? (in_col[i] && i != node) : !in_col[i];
    r.pend_tab_new[i] = keep ? (short)k : (short)-1;
    if (keep) {
      const int p = r.parent[i];
      parent_new[k] = (p >= 0 && r.pend_tab_new[p] >= 0) ? r.pend_tab_new[p] : (short)-1;
      fwd_new[k] = r.fwd[i];
      ++k;
    }
  }
  for (int i = r.T; i < SP_T; ++i) r.pend_tab_new[i] = -1;
  std::memcpy(r.parent, parent_new, sizeof(short) * k);
  std::memcpy(r.fwd, fwd_new, k);
  r.T = k;
  r.P += commit;
  *n_tab = k;
  *n_commit = commit;
}

// The mirror catches up with a prune that was decided on the device: waits for the copy of the verified
// node (queued right behind the kernel that produced it, so it has normally arrived long before any
// host code asks), then replays the prune on the parent list and returns the freed pages.
void reconcile(sp_stage* s, int req) {
  HostReq& r = s->reqs[req];
  if (!r.unrec) return;
  r.unrec = false;
  if (hipEventSynchronize(s->rec_ev) != hipSuccess) return;
  const int node = s->pin_nodes[r.unrec_slot];
  const int mode = (node >= 0 && node < r.T) ? SP_ACCEPT : SP_CLEAR;
  int live = 0, commit = 0;
  mirror_prune(r, mode, node, &live, &commit);
  r.pending = false;                               // the compaction was queued together with the prune
  if (is_paged(s->cfg)) (void)pages_resize(s, req, r.P + r.T, nullptr);
}

}  // namespace

extern "C" {

int sp_version(void) { return SP_VERSION; }

const char* sp_strerror(int status) {
  switch (status) {
    case SP_OK: return "ok";
    case SP_E_INVALID: return "invalid argument";
    case SP_E_CAPACITY: return "capacity exceeded";
    case SP_E_BAD_PARENT: return "bad parent index";
    case SP_E_BAD_REQ: return "bad or uninitialised request";
    case SP_E_BAD_NODE: return "bad node index";
    case SP_E_ORDER: return "parent not forwarded yet";
    case SP_E_PENDING: return "prune/compact out of order";
    case SP_E_HIP: return "HIP runtime error";
    case SP_E_UNSUPPORTED: return "unsupported shape or dtype";
    default: return "unknown status";
  }
}

int sp_last_hip_error(const sp_stage* stage) { return stage ? stage->last_hip : 0; }

int sp_stage_query_sizes(const sp_config* cfg, sp_sizes* out) {
  int rc = check_config(cfg);
  if (rc != SP_OK) return rc;
  if (!out) return SP_E_INVALID;
  const size_t row = (size_t)cfg->d_head * elt_bytes(cfg->dtype);
  out->kv_row_bytes = row;
  out->kv_plane_bytes = (size_t)cfg->kv_slots * row;
  out->kv_bytes = (size_t)cfg->n_layers * 2 * cfg->n_kv_heads * out->kv_plane_bytes;
  out->tables_bytes = tables_meta_bytes(*cfg) + align_up((size_t)cfg->max_requests * sizeof(ReqTables)) +
                      page_table_bytes(*cfg);
  out->workspace_bytes = carve(*cfg, nullptr).total;
  return SP_OK;
}

int sp_stage_create(const sp_config* cfg, const sp_layer_weights* layers, const sp_buffers* buffers,
                    sp_stream stream, sp_stage** out) {
  int rc = check_config(cfg);
  if (rc != SP_OK) return rc;
  if (!layers || !buffers || !out) return SP_E_INVALID;
  sp_sizes sz;
  sp_stage_query_sizes(cfg, &sz);
  if (!buffers->kv || !buffers->tables || !buffers->workspace) return SP_E_INVALID;
  if (buffers->kv_bytes < sz.kv_bytes || buffers->tables_bytes < sz.tables_bytes ||
      buffers->workspace_bytes < sz.workspace_bytes)
    return SP_E_CAPACITY;
  if (((uintptr_t)buffers->kv | (uintptr_t)buffers->tables | (uintptr_t)buffers->workspace) & 255) return SP_E_INVALID;
  for (int l = 0; l < cfg->n_layers; ++l) {
    const sp_layer_weights& w = layers[l];
    if (!w.wqkv || !w.wo || !w.wgu || !w.wd || !w.norm1 || !w.norm2) return SP_E_INVALID;
    if (((uintptr_t)w.wqkv | (uintptr_t)w.wo | (uintptr_t)w.wgu | (uintptr_t)w.wd) & 15) return SP_E_INVALID;
  }
  sp_stage* s = new (std::nothrow) sp_stage();
  if (!s) return SP_E_INVALID;
  s->cfg = *cfg;
  s->W.assign(layers, layers + cfg->n_layers);
  s->buf = *buffers;
  s->sizes = sz;
  s->d_meta = (ReqMeta*)buffers->tables;
  s->d_tables = (ReqTables*)((char*)buffers->tables + tables_meta_bytes(*cfg));
  s->ws = carve(*cfg, (char*)buffers->workspace);
  s->geom.kv = (char*)buffers->kv;
  s->geom.plane_bytes = sz.kv_plane_bytes;
  s->geom.row_bytes = (int)sz.kv_row_bytes;
  s->geom.n_layers = cfg->n_layers;
  s->geom.n_kv_heads = cfg->n_kv_heads;
  s->geom.page_table = nullptr; s->geom.pt_stride = 0; s->geom.pg_shift = 0;
  if (is_paged(*cfg)) {
    s->n_pages = (int)(cfg->kv_slots / cfg->page_slots);
    s->d_page_table = (int*)((char*)buffers->tables + tables_meta_bytes(*cfg) +
                             align_up((size_t)cfg->max_requests * sizeof(ReqTables)));
    s->geom.page_table = s->d_page_table;
    s->geom.pt_stride = s->n_pages;
    while ((1 << s->geom.pg_shift) < cfg->page_slots) ++s->geom.pg_shift;
    s->free_pages.resize(s->n_pages);
    for (int i = 0; i < s->n_pages; ++i) s->free_pages[i] = s->n_pages - 1 - i;    // page 0 is handed out first
  }
  s->reqs.resize(cfg->max_requests);
  // The MFMA kernels cover bf16 with d_head 128 and dimensions that fill their tiles.
  s->fast = cfg->dtype == SP_BF16 && !(cfg->flags & SP_FLAG_SIMPLE_KERNELS) && cfg->d_head == 128 &&
            cfg->d_model % 256 == 0 && cfg->d_ff % 256 == 0 &&
            (cfg->n_q_heads * cfg->d_head) % 256 == 0;
  {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= SP_NOALLOC_MAX_DEVICES) { delete s; return SP_E_HIP; }
    s->device = dev;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0)
      s->n_cu = cus;
    s->o_resident = (size_t)cfg->n_layers * cfg->d_model * cfg->n_q_heads * cfg->d_head * 2 <= ((size_t)128 << 20);
    if (!g_noalloc_scratch[dev]) {
      // this device's copy of the static scratch array (the device is current here)
      void* p = nullptr;
      if (hipGetSymbolAddress(&p, HIP_SYMBOL(sp_noalloc_scratch)) != hipSuccess || !p) { delete s; return SP_E_HIP; }
      g_noalloc_scratch[dev] = p;
    }
  }
  s->use_graphs = !(cfg->flags & SP_FLAG_NO_GRAPHS);
  s->packed = (cfg->flags & SP_FLAG_PACKED_WEIGHTS) != 0;
  if (s->packed && !s->fast) { delete s; return SP_E_UNSUPPORTED; }
  hipError_t e = sp_launch_tables_clear(s->d_meta, s->d_tables, cfg->max_requests, (hipStream_t)stream);
  if (e != hipSuccess) { delete s; return SP_E_HIP; }
  *out = s;
  return SP_OK;
}

void sp_stage_destroy(sp_stage* stage) {
  if (!stage) return;
  for (hipEvent_t ev : stage->prof_ev) (void)hipEventDestroy(ev);
  for (auto& g : stage->graphs) if (g.exec) (void)hipGraphExecDestroy(g.exec);
  if (stage->rec_ev) (void)hipEventDestroy(stage->rec_ev);
  if (stage->pin_nodes) (void)hipHostFree(stage->pin_nodes);
  delete stage;
}

int sp_pack_weights(const sp_config* cfg, const sp_layer_weights* in, const sp_layer_weights* out, sp_stream stream) {
  int rc = check_config(cfg);
  if (rc != SP_OK) return rc;
  if (!in || !out) return SP_E_INVALID;
  if (cfg->dtype != SP_BF16 || cfg->d_model % 32 || cfg->d_ff % 32 || cfg->d_head % 16) return SP_E_UNSUPPORTED;
  const int dq = cfg->n_q_heads * cfg->d_head, nqkv = (cfg->n_q_heads + 2 * cfg->n_kv_heads) * cfg->d_head;
  hipStream_t st = (hipStream_t)stream;
  if (!in->wqkv || !in->wo || !in->wgu || !in->wd || !out->wqkv || !out->wo || !out->wgu || !out->wd) return SP_E_INVALID;
  if (sp_launch_pack_weights(in->wqkv, (void*)out->wqkv, nqkv, cfg->d_model, st) != hipSuccess ||
      sp_launch_pack_weights(in->wo, (void*)out->wo, cfg->d_model, dq, st) != hipSuccess ||
      sp_launch_pack_weights(in->wgu, (void*)out->wgu, 2 * cfg->d_ff, cfg->d_model, st) != hipSuccess ||
      sp_launch_pack_weights(in->wd, (void*)out->wd, cfg->d_model, cfg->d_ff, st) != hipSuccess)
    return SP_E_HIP;
  return SP_OK;
}

int sp_pack_matrix(const void* in, void* out, int32_t n_rows, int32_t n_cols, sp_stream stream) {
  if (!in || !out || in == out || n_rows < 1 || n_cols < 1) return SP_E_INVALID;
  if (n_rows % 16 || n_cols % 32) return SP_E_UNSUPPORTED;
  return sp_launch_pack_weights(in, out, n_rows, n_cols, (hipStream_t)stream) == hipSuccess ? SP_OK : SP_E_HIP;
}

int sp_request_init(sp_stage* s, int32_t req, int64_t slot_base, int32_t capacity, int32_t prefix_len,
                    sp_stream stream) {
  if (!s) return SP_E_INVALID;
  if (req < 0 || req >= (int)s->reqs.size()) return SP_E_BAD_REQ;
  if (slot_base < 0 || capacity < 1 || prefix_len < 1) return SP_E_INVALID;
  // a reset does not care how a device-side prune of the old tree came out (its pages all go back below)
  s->reqs[req].unrec = false;
  HostReq& r = s->reqs[req];
  const bool paged = is_paged(s->cfg);
  if (paged) {
    // logical slots 0 .. capacity-1 on pages taken as the request grows; slot_base has no meaning
    if (slot_base != 0) return SP_E_INVALID;
    if (prefix_len > capacity || capacity > s->cfg.kv_slots) return SP_E_CAPACITY;
    if (pages_for(s, prefix_len) > (int)(s->free_pages.size() + r.pages.size())) return SP_E_CAPACITY;
  } else if (prefix_len > capacity || slot_base + capacity > s->cfg.kv_slots) {
    return SP_E_CAPACITY;
  }
  hipError_t e = sp_launch_request_init(s->d_meta, s->d_tables, req, slot_base, capacity, prefix_len,
                                        (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(s, e);
  if (paged) {
    if ((e = pages_resize(s, req, 0, (hipStream_t)stream)) != hipSuccess ||
        (e = pages_resize(s, req, prefix_len, (hipStream_t)stream)) != hipSuccess)
      return hip_fail(s, e);
  }
  r.active = true; r.base = slot_base; r.cap = capacity; r.P = prefix_len; r.T = 0; r.pending = false;
  r.unrec = false;
  return SP_OK;
}

int sp_request_release(sp_stage* s, int32_t req, sp_stream stream) {
  if (!s) return SP_E_INVALID;
  HostReq* r = get_req(s, req);
  if (!r) return SP_E_BAD_REQ;
  hipError_t e = is_paged(s->cfg) ? pages_resize(s, req, 0, (hipStream_t)stream) : hipSuccess;
  r->active = false; r->pending = false; r->T = 0; r->P = 0;
  return e == hipSuccess ? SP_OK : hip_fail(s, e);
}

int sp_request_pages(const sp_stage* s, int32_t req, int32_t* pages_out, int32_t max_pages, int32_t* n_pages_out) {
  if (!s || req < 0 || req >= (int)s->reqs.size() || !s->reqs[req].active) return s ? SP_E_BAD_REQ : SP_E_INVALID;
  if (s->reqs[req].unrec) reconcile(const_cast<sp_stage*>(s), req);
  if (!is_paged(s->cfg)) return SP_E_UNSUPPORTED;
  const HostReq& r = s->reqs[req];
  if (n_pages_out) *n_pages_out = (int32_t)r.pages.size();
  if (pages_out) {
    if (max_pages < (int)r.pages.size()) return SP_E_CAPACITY;
    for (size_t i = 0; i < r.pages.size(); ++i) pages_out[i] = r.pages[i];
  }
  return SP_OK;
}

int sp_stage_free_pages(const sp_stage* s) {
  if (!s) return SP_E_INVALID;
  for (size_t r = 0; r < s->reqs.size(); ++r)
    if (s->reqs[r].active && s->reqs[r].unrec) reconcile(const_cast<sp_stage*>(s), (int)r);
  return (int)s->free_pages.size();
}

int sp_request_info(const sp_stage* s, int32_t req, int32_t* prefix_len, int32_t* n_live, int32_t* n_forwarded) {
  if (!s) return SP_E_INVALID;
  if (req < 0 || req >= (int)s->reqs.size() || !s->reqs[req].active) return SP_E_BAD_REQ;
  if (s->reqs[req].unrec) reconcile(const_cast<sp_stage*>(s), req);
  const HostReq& r = s->reqs[req];
  if (prefix_len) *prefix_len = r.P;
  if (n_live) *n_live = r.T;
  if (n_forwarded) { int f = 0; for (int i = 0; i < r.T; ++i) f += r.fwd[i]; *n_forwarded = f; }
  return SP_OK;
}

int sp_tree_insert_batch(sp_stage* s, int32_t n_req, const int32_t* req_ids, const int32_t* n_new,
                         const int32_t* parents, const int32_t* tokens, const float* probs,
                         int32_t* first_index_out, sp_stream stream) {
  if (!s || !req_ids || !n_new) return SP_E_INVALID;
  if (n_req < 0 || n_req > SP_MAX_BATCH_REQ) return SP_E_CAPACITY;
  // validate everything before anything changes
  int total = 0;
  for (int i = 0; i < n_req; ++i) {
    HostReq* r = get_req(s, req_ids[i]);
    if (!r) return SP_E_BAD_REQ;
    if (n_new[i] < 0) return SP_E_INVALID;
    if (r->pending) return SP_E_PENDING;
    for (int j = 0; j < i; ++j) if (req_ids[j] == req_ids[i]) return SP_E_INVALID;
    if (r->T + n_new[i] > s->cfg.max_tree_nodes || r->P + r->T + n_new[i] > r->cap) return SP_E_CAPACITY;
    if (n_new[i] > 0 && !parents) return SP_E_INVALID;
    for (int k = 0; k < n_new[i]; ++k)
      if (parents[total + k] < -1 || parents[total + k] >= r->T + k) return SP_E_BAD_PARENT;
    total += n_new[i];
  }
  hipStream_t st = (hipStream_t)stream;
  if (is_paged(s->cfg)) {
    // pages for the new cache rows, all or nothing
    int need = 0;
    for (int i = 0; i < n_req; ++i) {
      const HostReq& r = s->reqs[req_ids[i]];
      need += pages_for(s, r.P + r.T + n_new[i]) - (int)r.pages.size();
    }
    if (need > (int)s->free_pages.size()) return SP_E_CAPACITY;
    for (int i = 0; i < n_req; ++i) {
      const HostReq& r = s->reqs[req_ids[i]];
      if (pages_for(s, r.P + r.T + n_new[i]) > (int)r.pages.size()) {
        hipError_t e = pages_resize(s, req_ids[i], r.P + r.T + n_new[i], st);
        if (e != hipSuccess) return hip_fail(s, e);
      }
    }
  }
  // launches of at most SP_T new nodes each (one launch in every case the configs produce)
  InsertArgs a;
  a.n_req = 0;
  a.row0[0] = 0;
  int row = 0;
  auto flush = [&]() -> hipError_t {
    if (a.n_req == 0) return hipSuccess;
    ProfScope scope(s, SP_K_TREE_INSERT, st);
    hipError_t e = sp_launch_tree_insert(s->d_meta, s->d_tables, a, s->geom, st);
    a.n_req = 0;
    a.row0[0] = 0;
    return e;
  };
  for (int i = 0; i < n_req; ++i) {
    HostReq& r = s->reqs[req_ids[i]];
    if (first_index_out) first_index_out[i] = r.T;
    const int n = n_new[i];
    if (n > 0) {
      if (a.row0[a.n_req] + n > SP_T) {
        hipError_t e = flush();
        if (e != hipSuccess) return hip_fail(s, e);
      }
      const int r0 = a.row0[a.n_req];
      a.req[a.n_req] = (short)req_ids[i];
      a.t0[a.n_req] = (short)r.T;
      a.first_slot[a.n_req] = r.base + r.P + r.T;
      for (int k = 0; k < n; ++k) {
        a.parent[r0 + k] = (short)parents[row + k];
        a.token[r0 + k] = tokens ? tokens[row + k] : 0;
        a.prob[r0 + k] = probs ? probs[row + k] : 0.f;
        r.parent[r.T + k] = (short)parents[row + k];
        r.fwd[r.T + k] = 0;
      }
      r.T += n;
      a.row0[++a.n_req] = (short)(r0 + n);
    }
    row += n;
  }
  hipError_t e = flush();
  return e == hipSuccess ? SP_OK : hip_fail(s, e);
}

int sp_tree_insert(sp_stage* s, int32_t req, int32_t n_new, const int32_t* parents, const int32_t* tokens,
                   const float* probs, int32_t* first_index_out, sp_stream stream) {
  if (!s) return SP_E_INVALID;
  return sp_tree_insert_batch(s, 1, &req, &n_new, parents, tokens, probs, first_index_out, stream);
}

int sp_stage_forward(sp_stage* s, int32_t n_req, const int32_t* req_ids, const int32_t* first_node,
                     const int32_t* n_nodes, const void* x_in, void* x_out, sp_stream stream) {
  if (!s || !req_ids || !first_node || !n_nodes) return SP_E_INVALID;
  if (n_req < 0 || n_req > SP_MAX_BATCH_REQ) return SP_E_CAPACITY;
  const sp_config& c = s->cfg;
  hipStream_t st = (hipStream_t)stream;
  FwdBatch b;
  b.n_req = 0;
  int rows = 0;
  for (int i = 0; i < n_req; ++i) {
    HostReq* r = get_req(s, req_ids[i]);
    if (!r) return SP_E_BAD_REQ;
    if (r->pending) return SP_E_PENDING;
    for (int j = 0; j < i; ++j) if (req_ids[j] == req_ids[i]) return SP_E_INVALID;
    if (n_nodes[i] < 0) return SP_E_INVALID;
    if (n_nodes[i] == 0) continue;
    if (first_node[i] < 0 || first_node[i] + n_nodes[i] > r->T) return SP_E_BAD_NODE;
    for (int k = first_node[i]; k < first_node[i] + n_nodes[i]; ++k) {
      const int p = r->parent[k];
      if (p >= 0 && !r->fwd[p] && p < first_node[i]) return SP_E_ORDER;
    }
    b.req[b.n_req] = req_ids[i]; b.first[b.n_req] = first_node[i]; b.n[b.n_req] = n_nodes[i]; b.row0[b.n_req] = rows;
    ++b.n_req;
    rows += n_nodes[i];
  }
  if (rows > c.max_batch_nodes) return SP_E_CAPACITY;
  if (rows == 0) return SP_OK;
  if (!x_in || !x_out) return SP_E_INVALID;
  b.n_rows = rows;
  const int M = rows, d = c.d_model, F = c.d_ff, dh = c.d_head, nq = c.n_q_heads, nkv = c.n_kv_heads;
  const int dq = nq * dh, nqkv = (nq + 2 * nkv) * dh;
  const int dt = c.dtype;
  Workspace& w = s->ws;
  hipError_t e;
#define SP_TRY(call) do { e = (call); if (e != hipSuccess) return hip_fail(s, e); } while (0)

  AttnPlan plan;
  std::memset(&plan, 0, sizeof(plan));
  plan.n_seg = b.n_req;
  for (int i = 0; i < b.n_req; ++i) {              // which request and node each row belongs to
    const HostReq& r = s->reqs[b.req[i]];
    plan.seg_row0[i] = b.row0[i]; plan.seg_rows[i] = b.n[i]; plan.seg_req[i] = b.req[i];
    plan.seg_first[i] = b.first[i]; plan.seg_P[i] = r.P; plan.seg_T[i] = r.T; plan.seg_base[i] = r.base;
    plan.seg_chunks[i] = 1;
  }
  if (s->fast) {
    // Split every request's cache range into chunks so that the grid fills the chip
    // and the partial results fit the workspace.
    const int g = nq / nkv;
    int maxq = 0;
    for (int i = 0; i < b.n_req; ++i) if (b.n[i] * g > maxq) maxq = b.n[i] * g;
    plan.qt = maxq <= 16 ? 1 : 2;
    const int qrows_per_block = 16 * plan.qt;
    // One workgroup per CU is the target.  If the query blocks alone give that many, every
    // request keeps its whole cache range in one chunk (no partial results, no merge kernel);
    // otherwise each range is cut into `want` chunks, but never below one 32-slot tile per
    // wave, and fewer if the partial results would not fit the workspace.
    auto fill = [&](int want, size_t* units_out) {
      size_t units = 0; int items = 0, split = 0;
      for (int i = 0; i < b.n_req; ++i) {
        const HostReq& r = s->reqs[b.req[i]];
        const int span = r.P + r.T;
        int chunks = want;
        const int max_chunks = (span + 255) / 256;
        if (chunks > max_chunks) chunks = max_chunks;
        if (chunks < 1) chunks = 1;
        const int clen = ((span + chunks - 1) / chunks + 31) / 32 * 32;
        chunks = (span + clen - 1) / clen;
        const int qblocks = (b.n[i] * g + qrows_per_block - 1) / qrows_per_block;
        plan.seg_item0[i] = items; plan.seg_chunks[i] = chunks; plan.seg_clen[i] = clen; plan.seg_qblocks[i] = qblocks;
        plan.seg_unit0[i] = (int)units;
        items += chunks * qblocks;
        if (chunks > 1) { units += (size_t)chunks * b.n[i] * nq; split = 1; }
      }
      plan.seg_item0[b.n_req] = items;
      plan.total_items = items;
      plan.units_total = (int)units;
      plan.any_split = split;
      *units_out = units;
      return items;
    };
    int base_blocks = 0;
    for (int i = 0; i < b.n_req; ++i) base_blocks += (b.n[i] * g + qrows_per_block - 1) / qrows_per_block;
    int want = s->n_cu / (base_blocks * nkv);
    size_t units = 0;
    fill(want, &units);
    while (units > w.attn_units && want > 1) { want = (want + 1) / 2; fill(want, &units); }
    if (units > w.attn_units) return SP_E_CAPACITY;
  }

  const size_t strideD = (size_t)M * d, strideQ = (size_t)M * nqkv;
  // projections: few rows stream the weights (HBM-bound); many rows use the register-blocked kernel
  const bool wide = s->fast && M > 128 && nqkv % 256 == 0 && d % 256 == 0 && F % 128 == 0 && dq % 128 == 0;
  auto gemm = [&](const void* X, const void* Wm, int N_, int K_, int* S_, bool resident = false) -> hipError_t {
    if (wide)
      return sp_launch_gemm_wide((const bf16_t*)X, (const bf16_t*)Wm, s->packed, w.part, M, N_, K_, s->n_cu,
                                 w.part_floats, S_, st);
    return sp_launch_gemm_bf16((const bf16_t*)X, (const bf16_t*)Wm, s->packed, w.part, M, N_, K_, 16, w.part_floats,
                               S_, st, resident);
  };
  // Everything between the kernel that opens the call (rows enter, first RMSNorm, plan to device
  // memory) and the one that writes the result out.  No argument of these launches depends on the
  // caller's pointers or on the plan's contents, only on M and on the grid sizes the plan implies.
  int S_last = 0;
#define SP_STEP(call) do { hipError_t e_ = (call); if (e_ != hipSuccess) return e_; } while (0)
  auto run_layers = [&]() -> hipError_t {
    int S_prev = 0;                                 // split count of the previous layer's down projection
    for (int l = 0; l < c.n_layers; ++l) {
      const sp_layer_weights& L = s->W[l];
      if (l > 0) {
        ProfScope p(s, SP_K_NORM, st);
        SP_STEP(sp_launch_add_norm(dt, w.h, w.part, S_prev, strideD, L.norm1, w.xn, M, d, c.rms_eps, st));
      }
      int S = 1;
      { ProfScope p(s, SP_K_GEMM_QKV, st);
        if (s->fast) SP_STEP(gemm(w.xn, L.wqkv, nqkv, d, &S));
        else SP_STEP(sp_launch_gemm_simple(dt, w.xn, L.wqkv, w.part, M, nqkv, d, st)); }
      { ProfScope p(s, SP_K_ROPE_KV, st);
        SP_STEP(sp_launch_rope_kv(dt, w.part, S, strideQ, w.rows, w.cs, w.qbuf, s->geom, l, M, nq, nkv, dh, st)); }
      if (s->fast) {
        ProfScope p(s, SP_K_ATTENTION, st);
        SP_STEP(sp_launch_attn_bf16((const bf16_t*)w.qbuf, s->d_tables, s->geom, l, plan, w.plan, w.attn_part,
                                    (bf16_t*)w.attn, M, nq, nkv, dh, st));
      } else {
        ProfScope p(s, SP_K_ATTENTION, st);
        SP_STEP(sp_launch_attn_simple(dt, w.qbuf, w.rows, s->d_tables, s->geom, l, w.attn, M, nq, nkv, dh, st));
      }
      { ProfScope p(s, SP_K_GEMM_O, st);
        S = 1;
        if (s->fast) SP_STEP(gemm(w.attn, L.wo, d, dq, &S, s->o_resident));
        else SP_STEP(sp_launch_gemm_simple(dt, w.attn, L.wo, w.part, M, d, dq, st)); }
      { ProfScope p(s, SP_K_NORM, st);
        SP_STEP(sp_launch_add_norm(dt, w.h, w.part, S, strideD, L.norm2, w.xn, M, d, c.rms_eps, st)); }
      { ProfScope p(s, SP_K_GEMM_GATEUP, st);
        if (s->fast) {
          if (wide) SP_STEP(sp_launch_gemm_wide_gateup((const bf16_t*)w.xn, (const bf16_t*)L.wgu, s->packed, (bf16_t*)w.act, M, F, d, st));
          else SP_STEP(sp_launch_gemm_gateup_bf16((const bf16_t*)w.xn, (const bf16_t*)L.wgu, s->packed, (bf16_t*)w.act, M, F, d, s->n_cu, st));
        } else {
          SP_STEP(sp_launch_gemm_simple(dt, w.xn, L.wgu, w.part, M, 2 * F, d, st));
          SP_STEP(sp_launch_silu_mul(dt, w.part, w.act, M, F, st));
        } }
      { ProfScope p(s, SP_K_GEMM_DOWN, st);
        S = 1;
        if (s->fast) SP_STEP(gemm(w.act, L.wd, d, F, &S));
        else SP_STEP(sp_launch_gemm_simple(dt, w.act, L.wd, w.part, M, d, F, st)); }
      S_prev = S;
    }
    S_last = S_prev;
    return hipSuccess;
  };
#undef SP_STEP

  { ProfScope p(s, SP_K_NORM, st);
    SP_TRY(sp_launch_enter_norm(dt, x_in, plan, s->fast ? w.plan : nullptr, s->d_meta, s->d_tables, w.rows, w.cs, dh,
                                c.rope_theta, w.h, s->W[0].norm1, w.xn, M, d, c.rms_eps, st)); }

  // A shape that comes back replays its graph; one seen for the second time is captured.  Not while a
  // kernel kind is being timed (the events sit between the launches) and not inside a caller's capture.
  sp_stage::FwdGraph* fg = nullptr;
  bool timed = false;                               // an event bracket falls inside this call's layers
  int n_kind = 0;                                   // launches of the timed kind among them
  if (s->prof_kind != 0) {
    const int k = s->prof_kind;
    if (k == SP_K_GEMM_QKV || k == SP_K_GEMM_O || k == SP_K_GEMM_GATEUP || k == SP_K_GEMM_DOWN ||
        k == SP_K_ATTENTION || k == SP_K_ROPE_KV) n_kind = c.n_layers;
    else if (k == SP_K_NORM) n_kind = 2 * c.n_layers - 1;
    if (n_kind > 0) {
      // whole calls are sampled: align the count to this call's group of launches
      s->prof_group = n_kind;
      s->prof_seen = (s->prof_seen + n_kind - 1) / n_kind * n_kind;
      timed = s->prof_n < s->prof_max && ((s->prof_seen / n_kind) % s->prof_every) == 0;
    }
  }
  if (s->use_graphs && s->fast && !timed) {
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(st, &cap) == hipSuccess && cap == hipStreamCaptureStatusNone) {
      for (auto& g : s->graphs)
        if (g.M == M && g.qt == plan.qt && g.items == plan.total_items && g.any_split == plan.any_split &&
            g.units == plan.units_total) { fg = &g; break; }
      if (!fg && s->graphs.size() < 256) {
        s->graphs.push_back({M, plan.qt, plan.total_items, plan.any_split, plan.units_total, 0, 0, false, nullptr});
        fg = &s->graphs.back();
      }
    }
  }
  bool done = false;
  if (fg) {
    ++fg->seen;
    const int seen_before = s->prof_seen;
    if (!fg->exec && !fg->failed && fg->seen >= 2) {
      hipGraph_t graph = nullptr;
      if (hipStreamBeginCapture(st, hipStreamCaptureModeThreadLocal) == hipSuccess) {
        const hipError_t e_run = run_layers();
        const hipError_t e_end = hipStreamEndCapture(st, &graph);
        if (e_run == hipSuccess && e_end == hipSuccess && graph &&
            hipGraphInstantiate(&fg->exec, graph, nullptr, nullptr, 0) == hipSuccess) {
          fg->S_last = S_last;
        } else {
          fg->exec = nullptr;
          fg->failed = true;
          (void)hipGetLastError();
        }
        if (graph) (void)hipGraphDestroy(graph);
      } else {
        fg->failed = true;
        (void)hipGetLastError();
      }
    }
    if (fg->exec) {
      SP_TRY(hipGraphLaunch(fg->exec, st));
      S_last = fg->S_last;
      // the sampling cadence counts the replayed launches too (once: the capturing call has already
      // counted them while it recorded the launches)
      s->prof_seen = seen_before + n_kind;
      done = true;
    }
  }
  if (!done) SP_TRY(run_layers());
  SP_TRY(sp_launch_finish(dt, w.h, w.part, S_last, strideD, x_out, M, d, st));
#undef SP_TRY
  for (int i = 0; i < b.n_req; ++i) {
    HostReq& r = s->reqs[b.req[i]];
    for (int k = b.first[i]; k < b.first[i] + b.n[i]; ++k) r.fwd[k] = 1;
  }
  return SP_OK;
}

int sp_tree_prune_batch(sp_stage* s, int32_t n, const int32_t* req_ids, const int32_t* modes, const int32_t* nodes,
                        int32_t* n_live_out, int32_t* n_commit_out, sp_stream stream) {
  if (!s || !req_ids || !modes || !nodes) return SP_E_INVALID;
  if (n < 0 || n > SP_MAX_BATCH_REQ) return SP_E_CAPACITY;
  PruneBatch b;
  b.n = n;
  bool any = false;
  for (int i = 0; i < n; ++i) {
    b.req[i] = req_ids[i]; b.mode[i] = modes[i]; b.node[i] = nodes[i];
    if (modes[i] < 0) continue;
    HostReq* r = get_req(s, req_ids[i]);
    if (!r) return SP_E_BAD_REQ;
    if (modes[i] != SP_ACCEPT && modes[i] != SP_DROP && modes[i] != SP_CLEAR) return SP_E_INVALID;
    if (r->pending) return SP_E_PENDING;
    if (modes[i] != SP_CLEAR && (nodes[i] < 0 || nodes[i] >= r->T)) return SP_E_BAD_NODE;
    if (modes[i] == SP_ACCEPT)
      // the path root..node joins the committed context: its K/V rows must exist at this stage
      for (int j = nodes[i]; j >= 0; j = r->parent[j]) if (!r->fwd[j]) return SP_E_ORDER;
    for (int j = 0; j < i; ++j) if (modes[j] >= 0 && req_ids[j] == req_ids[i]) return SP_E_INVALID;
    any = true;
  }
  if (any) {
    hipError_t e = sp_launch_tree_prune(s->d_meta, s->d_tables, b, nullptr, 0, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(s, e);
  }
  for (int i = 0; i < n; ++i) {
    int live = 0, commit = 0;
    if (modes[i] >= 0) {
      HostReq& r = s->reqs[req_ids[i]];
      r.pend_mode = modes[i]; r.pend_node = nodes[i];
      mirror_prune(r, modes[i], nodes[i], &live, &commit);
      r.pending = true;
    } else if (HostReq* r = get_req(s, req_ids[i])) {
      live = r->T;
    }
    if (n_live_out) n_live_out[i] = live;
    if (n_commit_out) n_commit_out[i] = commit;
  }
  return SP_OK;
}

int sp_tree_prune(sp_stage* s, int32_t req, int32_t mode, int32_t node, int32_t* n_live_out, int32_t* n_commit_out,
                  sp_stream stream) {
  if (mode < 0) return SP_E_INVALID;
  if (!s) return SP_E_INVALID;
  ProfScope scope(s, SP_K_TREE_PRUNE, (hipStream_t)stream);
  return sp_tree_prune_batch(s, 1, &req, &mode, &node, n_live_out, n_commit_out, stream);
}

int sp_tree_prune_verified(sp_stage* s, int32_t n, const int32_t* req_ids, const int32_t* nodes_dev, int32_t stride,
                           sp_stream stream) {
  if (!s || !req_ids || !nodes_dev) return SP_E_INVALID;
  if (n < 0 || n > SP_MAX_BATCH_REQ) return SP_E_CAPACITY;
  if (stride < 1 || stride > 2) return SP_E_INVALID;
  PruneBatch b;
  b.n = n;
  for (int i = 0; i < n; ++i) {
    HostReq* r = get_req(s, req_ids[i]);                  // (takes in any earlier device-side prune of the request)
    if (!r) return SP_E_BAD_REQ;
    if (r->pending) return SP_E_PENDING;
    for (int j = 0; j < i; ++j) if (req_ids[j] == req_ids[i]) return SP_E_INVALID;
    b.req[i] = req_ids[i]; b.mode[i] = SP_ACCEPT; b.node[i] = 0;
  }
  if (n == 0) return SP_OK;
  // one batch of results is in flight at a time: the pinned buffer is free once every request of the
  // previous batch has been taken in
  for (size_t q = 0; q < s->reqs.size(); ++q) if (s->reqs[q].active && s->reqs[q].unrec) reconcile(s, (int)q);
  hipError_t e;
  if (!s->pin_nodes) {
    if ((e = hipHostMalloc((void**)&s->pin_nodes, sizeof(int) * 2 * SP_MAX_BATCH_REQ, hipHostMallocDefault)) != hipSuccess)
      return hip_fail(s, e);
    if ((e = hipEventCreateWithFlags(&s->rec_ev, hipEventDisableTiming)) != hipSuccess) return hip_fail(s, e);
  }
  hipStream_t st = (hipStream_t)stream;
  { ProfScope scope(s, SP_K_TREE_PRUNE, st);
    if ((e = sp_launch_tree_prune(s->d_meta, s->d_tables, b, nodes_dev, stride, st)) != hipSuccess) return hip_fail(s, e); }
  { ProfScope scope(s, SP_K_KV_COMPACT, st);
    const size_t rb = (size_t)s->cfg.d_model * elt_bytes(s->cfg.dtype);
    if ((e = sp_launch_kv_compact(s->d_meta, s->d_tables, b, s->geom, nullptr, rb, (int)rb, nullptr, st)) != hipSuccess)
      return hip_fail(s, e); }
  if ((e = hipMemcpyAsync(s->pin_nodes, nodes_dev, sizeof(int) * (size_t)n * stride, hipMemcpyDeviceToHost, st)) != hipSuccess ||
      (e = hipEventRecord(s->rec_ev, st)) != hipSuccess)
    return hip_fail(s, e);
  for (int i = 0; i < n; ++i) {
    HostReq& r = s->reqs[req_ids[i]];
    r.unrec = true;
    r.unrec_slot = i * stride;
  }
  return SP_OK;
}

// rows / list (nullable, one request only): hidden rows compacted by the same launch as the cache
static int compact_batch(sp_stage* s, int32_t n, const int32_t* req_ids, void* rows, const RowList* list,
                         sp_stream stream) {
  if (!s || !req_ids) return SP_E_INVALID;
  if (n < 0 || n > SP_MAX_BATCH_REQ) return SP_E_CAPACITY;
  PruneBatch b;
  b.n = n;
  for (int i = 0; i < n; ++i) {
    HostReq* r = get_req(s, req_ids[i]);
    if (!r) return SP_E_BAD_REQ;
    if (!r->pending) return SP_E_PENDING;
    for (int j = 0; j < i; ++j) if (req_ids[j] == req_ids[i]) return SP_E_INVALID;
    b.req[i] = req_ids[i]; b.mode[i] = r->pend_mode; b.node[i] = r->pend_node;
  }
  if (n == 0) return SP_OK;
  {
    ProfScope scope(s, SP_K_KV_COMPACT, (hipStream_t)stream);
    const size_t rb = (size_t)s->cfg.d_model * elt_bytes(s->cfg.dtype);
    hipError_t e = sp_launch_kv_compact(s->d_meta, s->d_tables, b, s->geom, rows, rb, (int)rb, list, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(s, e);
  }
  hipError_t e_pages = hipSuccess;
  for (int i = 0; i < n; ++i) {
    HostReq& r = s->reqs[req_ids[i]];
    r.pending = false;
    // pages past the compacted rows go back to the allocator (work queued later runs after the gather)
    if (is_paged(s->cfg)) {
      const hipError_t e = pages_resize(s, req_ids[i], r.P + r.T, (hipStream_t)stream);
      if (e != hipSuccess && e_pages == hipSuccess) e_pages = e;
    }
  }
  return e_pages == hipSuccess ? SP_OK : hip_fail(s, e_pages);
}

int sp_kv_compact_batch(sp_stage* s, int32_t n, const int32_t* req_ids, sp_stream stream) {
  return compact_batch(s, n, req_ids, nullptr, nullptr, stream);
}

int sp_kv_compact(sp_stage* s, int32_t req, void* x_rows, int32_t n_rows, const int32_t* row_nodes,
                  int32_t* n_rows_out, int32_t* row_nodes_out, sp_stream stream) {
  if (!s) return SP_E_INVALID;
  HostReq* r = get_req(s, req);
  if (!r) return SP_E_BAD_REQ;
  if (!r->pending) return SP_E_PENDING;
  RowList list;
  list.n_keep = 0;
  list.first_moved = 0;
  if (x_rows) {
    if (n_rows < 0 || n_rows > SP_T || (n_rows > 0 && !row_nodes)) return SP_E_INVALID;
    bool moved = false;
    for (int i = 0; i < n_rows; ++i) {
      const int node = row_nodes[i];
      if (node < 0 || node >= SP_T) return SP_E_BAD_NODE;
      if (i > 0 && node <= row_nodes[i - 1]) return SP_E_INVALID;
      int nn;
      bool keep;
      if (r->pend_mode == SP_ACCEPT && node == r->pend_node) { keep = true; nn = -1; }
      else { nn = r->pend_tab_new[node]; keep = nn >= 0; }
      if (keep) {
        if (!moved && i != list.n_keep) { moved = true; list.first_moved = list.n_keep; }
        list.src[list.n_keep] = (short)i;
        if (row_nodes_out) row_nodes_out[list.n_keep] = nn;
        ++list.n_keep;
      }
    }
    if (!moved) list.first_moved = list.n_keep;
  }
  const bool move_rows = x_rows && list.first_moved < list.n_keep;
  int rc = compact_batch(s, 1, &req, move_rows ? x_rows : nullptr, move_rows ? &list : nullptr, stream);
  if (rc != SP_OK) return rc;
  if (x_rows) {
    if (n_rows_out) *n_rows_out = list.n_keep;
  } else if (n_rows_out) {
    *n_rows_out = 0;
  }
  return SP_OK;
}

int sp_tree_read(sp_stage* s, int32_t req, sp_tree_view* out, sp_stream stream) {
  if (!s || !out) return SP_E_INVALID;
  if (!get_req(s, req)) return SP_E_BAD_REQ;
  hipStream_t st = (hipStream_t)stream;
  ReqMeta m;
  hipError_t e = hipMemcpyAsync(&m, s->d_meta + req, sizeof(ReqMeta), hipMemcpyDeviceToHost, st);
  if (e != hipSuccess) return hip_fail(s, e);
  const ReqTables* t = s->d_tables + req;
  if ((e = hipMemcpyAsync(out->parent, t->parent, sizeof(out->parent), hipMemcpyDeviceToHost, st)) != hipSuccess ||
      (e = hipMemcpyAsync(out->depth, t->depth, sizeof(out->depth), hipMemcpyDeviceToHost, st)) != hipSuccess ||
      (e = hipMemcpyAsync(out->token, t->token, sizeof(out->token), hipMemcpyDeviceToHost, st)) != hipSuccess ||
      (e = hipMemcpyAsync(out->prob, t->prob, sizeof(out->prob), hipMemcpyDeviceToHost, st)) != hipSuccess ||
      (e = hipMemcpyAsync(out->pred, t->pred, sizeof(out->pred), hipMemcpyDeviceToHost, st)) != hipSuccess ||
      (e = hipMemcpyAsync(out->anc, t->anc, sizeof(out->anc), hipMemcpyDeviceToHost, st)) != hipSuccess)
    return hip_fail(s, e);
  if ((e = hipStreamSynchronize(st)) != hipSuccess) return hip_fail(s, e);
  out->prefix_len = m.P;
  out->n_live = m.T;
  out->root_pred = m.root_pred;
  return SP_OK;
}

int sp_request_set_root_pred(sp_stage* s, int32_t req, int32_t token, sp_stream stream) {
  if (!s) return SP_E_INVALID;
  if (!get_req(s, req)) return SP_E_BAD_REQ;
  if (token < 0) return SP_E_INVALID;
  hipError_t e = sp_launch_set_root_pred(s->d_meta, req, token, (hipStream_t)stream);
  return e == hipSuccess ? SP_OK : hip_fail(s, e);
}

// Device buffers the output head works in: the stage's workspace, or the static scratch array.
struct HeadScratch {
  RowInfo* rows;
  float* cs;
  float* h;
  void* xn;
  float* part;
  size_t part_floats;
  int max_rows;
};

static int verify_head_on(sp_stage* s, const HeadScratch& w, const sp_head_weights* head, int32_t n_req,
                          const int32_t* req_ids, const int32_t* first_node, const int32_t* n_nodes, const void* x,
                          int32_t* pred_out, float* max_out, sp_stream stream) {
  if (!s || !head || !req_ids || !first_node || !n_nodes) return SP_E_INVALID;
  if (!head->norm || !head->wvocab || head->vocab < 1) return SP_E_INVALID;
  if (n_req < 0 || n_req > SP_MAX_BATCH_REQ) return SP_E_CAPACITY;
  const sp_config& c = s->cfg;
  hipStream_t st = (hipStream_t)stream;
  FwdBatch b;
  b.n_req = 0;
  int rows = 0;
  for (int i = 0; i < n_req; ++i) {
    HostReq* r = get_req(s, req_ids[i]);
    if (!r) return SP_E_BAD_REQ;
    if (r->pending) return SP_E_PENDING;
    for (int j = 0; j < i; ++j) if (req_ids[j] == req_ids[i]) return SP_E_INVALID;
    if (n_nodes[i] < 0) return SP_E_INVALID;
    if (n_nodes[i] == 0) continue;
    if (first_node[i] < 0 || first_node[i] + n_nodes[i] > r->T) return SP_E_BAD_NODE;
    // a prediction needs the node's output of the last layer: it must have been forwarded
    for (int k = first_node[i]; k < first_node[i] + n_nodes[i]; ++k) if (!r->fwd[k]) return SP_E_ORDER;
    b.req[b.n_req] = req_ids[i]; b.first[b.n_req] = first_node[i]; b.n[b.n_req] = n_nodes[i]; b.row0[b.n_req] = rows;
    ++b.n_req;
    rows += n_nodes[i];
  }
  if (rows > w.max_rows) return SP_E_CAPACITY;
  if (rows == 0) return SP_OK;
  if (!x) return SP_E_INVALID;
  b.n_rows = rows;
  const int M = rows, d = c.d_model, V = head->vocab;
  hipError_t e;
  // final RMSNorm (the row descriptors and the float copy of x it also writes are scratch here)
  AttnPlan rows_of;                                   // only the segment fields are read
  std::memset(&rows_of, 0, sizeof(rows_of));
  rows_of.n_seg = b.n_req;
  for (int i = 0; i < b.n_req; ++i) {
    rows_of.seg_row0[i] = b.row0[i]; rows_of.seg_rows[i] = b.n[i]; rows_of.seg_req[i] = b.req[i];
    rows_of.seg_first[i] = b.first[i];
  }
  e = sp_launch_enter_norm(c.dtype, x, rows_of, nullptr, s->d_meta, s->d_tables, w.rows, w.cs, c.d_head, c.rope_theta,
                           w.h, head->norm, w.xn, M, d, c.rms_eps, st);
  if (e != hipSuccess) return hip_fail(s, e);
  ProfScope p(s, SP_K_VERIFY_HEAD, st);
  if (s->fast && V % 64 == 0 && d % 128 == 0) {
    int tiles = 0;
    e = sp_launch_gemm_argmax_bf16((const bf16_t*)w.xn, (const bf16_t*)head->wvocab, s->packed, w.part, M, V, d,
                                   w.part_floats, &tiles, st);
    if (e == hipErrorInvalidValue) return SP_E_CAPACITY;
    if (e == hipSuccess) e = sp_launch_argmax_rows(true, w.part, tiles, b, s->d_tables, pred_out, max_out, st);
  } else {
    if ((size_t)M * V > w.part_floats) return SP_E_CAPACITY;
    e = sp_launch_gemm_simple(c.dtype, w.xn, head->wvocab, w.part, M, V, d, st);
    if (e == hipSuccess) e = sp_launch_argmax_rows(false, w.part, V, b, s->d_tables, pred_out, max_out, st);
  }
  return e == hipSuccess ? SP_OK : hip_fail(s, e);
}

int sp_stage_verify_head(sp_stage* s, const sp_head_weights* head, int32_t n_req, const int32_t* req_ids,
                         const int32_t* first_node, const int32_t* n_nodes, const void* x, int32_t* pred_out,
                         float* max_out, sp_stream stream) {
  if (!s) return SP_E_INVALID;
  const Workspace& ws = s->ws;
  const HeadScratch w = {ws.rows, ws.cs, ws.h, ws.xn, ws.part, ws.part_floats, s->cfg.max_batch_nodes};
  return verify_head_on(s, w, head, n_req, req_ids, first_node, n_nodes, x, pred_out, max_out, stream);
}

int sp_stage_verify_head_noalloc(sp_stage* s, const sp_head_weights* head, int32_t n_req, const int32_t* req_ids,
                                 const int32_t* first_node, const int32_t* n_nodes, const void* x,
                                 int32_t* pred_out, float* max_out, sp_stream stream) {
  if (!s) return SP_E_INVALID;
  char* base = (char*)g_noalloc_scratch[s->device];     // this device's copy, looked up at sp_stage_create
  if (!base) return SP_E_INVALID;
  const sp_config& c = s->cfg;
  // fixed carve for SP_NOALLOC_MAX_ROWS rows; whatever is left holds the (value, index) pairs or the logits
  const size_t R = SP_NOALLOC_MAX_ROWS;
  size_t off = 0;
  auto take = [&](size_t bytes) { char* p = base + off; off += align_up(bytes); return (void*)p; };
  HeadScratch w;
  w.rows = (RowInfo*)take(R * sizeof(RowInfo));
  w.cs = (float*)take(R * c.d_head * sizeof(float));
  w.h = (float*)take(R * c.d_model * sizeof(float));
  w.xn = take(R * c.d_model * (size_t)elt_bytes(c.dtype));
  if (off + 256 > SP_NOALLOC_SCRATCH_BYTES) return SP_E_CAPACITY;      // d_model too large for the array
  w.part = (float*)(base + off);
  w.part_floats = (SP_NOALLOC_SCRATCH_BYTES - off) / sizeof(float);
  w.max_rows = (int)R < c.max_batch_nodes ? (int)R : c.max_batch_nodes;
  return verify_head_on(s, w, head, n_req, req_ids, first_node, n_nodes, x, pred_out, max_out, stream);
}

int sp_stage_verify_lossy(sp_stage* s, const sp_head_weights* head, int32_t n, const int32_t* req_ids,
                          const void* x_root, int32_t mode, float top_p, int32_t* result_dev, int32_t* result_host,
                          sp_stream stream) {
  if (!s || !head || !req_ids || !result_dev) return SP_E_INVALID;
  if (!head->norm || !head->wvocab || head->vocab < 1) return SP_E_INVALID;
  if (mode != SP_VERIFY_RELAXED && mode != SP_VERIFY_TOP_P) return SP_E_INVALID;
  if (mode == SP_VERIFY_TOP_P && !(top_p > 0.f && top_p <= 1.f)) return SP_E_INVALID;   // also rejects NaN
  const sp_config& c = s->cfg;
  if (n < 0 || n > SP_MAX_BATCH_REQ || n > c.max_batch_nodes) return SP_E_CAPACITY;
  for (int i = 0; i < n; ++i) {
    HostReq* r = get_req(s, req_ids[i]);
    if (!r) return SP_E_BAD_REQ;
    if (r->pending) return SP_E_PENDING;
    for (int j = 0; j < i; ++j) if (req_ids[j] == req_ids[i]) return SP_E_INVALID;
  }
  if (n == 0) return SP_OK;
  if (!x_root) return SP_E_INVALID;
  const int d = c.d_model, V = head->vocab;
  Workspace& w = s->ws;
  const size_t logit_floats = (size_t)n * V;
  if (logit_floats + sp_lossy_scratch_floats(n, V) > w.part_floats) return SP_E_CAPACITY;
  hipStream_t st = (hipStream_t)stream;
  hipError_t e = sp_launch_row_norm(c.dtype, x_root, head->norm, w.xn, n, d, c.rms_eps, st);
  if (e != hipSuccess) return hip_fail(s, e);
  ProfScope p(s, SP_K_VERIFY_HEAD, st);
  if (s->fast && V % 64 == 0 && d % 128 == 0) {
    int S = 1;
    e = sp_launch_gemm_bf16((const bf16_t*)w.xn, (const bf16_t*)head->wvocab, s->packed, w.part, n, V, d, 1,
                            logit_floats, &S, st);
  } else {
    e = sp_launch_gemm_simple(c.dtype, w.xn, head->wvocab, w.part, n, V, d, st);
  }
  if (e == hipSuccess)
    e = sp_launch_verify_lossy(s->d_meta, s->d_tables, w.part, n, req_ids, V, mode, top_p, w.part + logit_floats,
                               result_dev, st);
  if (e == hipSuccess && result_host)
    e = hipMemcpyAsync(result_host, result_dev, sizeof(int32_t) * 2 * n, hipMemcpyDeviceToHost, st);
  return e == hipSuccess ? SP_OK : hip_fail(s, e);
}

int sp_stage_verify_sample(sp_stage* s, const sp_head_weights* head, int32_t n, const int32_t* req_ids,
                           const void* x_root, float temperature, float top_p, int32_t top_k, const float* u,
                           int32_t* result_dev, int32_t* result_host, sp_stream stream) {
  if (!s || !head || !req_ids || !result_dev || !u) return SP_E_INVALID;
  if (!head->norm || !head->wvocab || head->vocab < 1) return SP_E_INVALID;
  if (!(temperature > 0.f) || !(top_p > 0.f && top_p <= 1.f)) return SP_E_INVALID;      // also rejects NaN
  if (top_k < 1 || top_k > SP_MAX_SAMPLE_TOP_K) return SP_E_INVALID;
  const sp_config& c = s->cfg;
  if (n < 0 || n > SP_MAX_BATCH_REQ || n > c.max_batch_nodes) return SP_E_CAPACITY;
  for (int i = 0; i < n; ++i) {
    HostReq* r = get_req(s, req_ids[i]);
    if (!r) return SP_E_BAD_REQ;
    if (r->pending) return SP_E_PENDING;
    if (!(u[i] >= 0.f && u[i] < 1.f)) return SP_E_INVALID;
    for (int j = 0; j < i; ++j) if (req_ids[j] == req_ids[i]) return SP_E_INVALID;
  }
  if (n == 0) return SP_OK;
  if (!x_root) return SP_E_INVALID;
  const int d = c.d_model, V = head->vocab;
  if (V >= (1 << 16) * 1024) return SP_E_UNSUPPORTED;                  // the gather counts 16 bits per thread
  Workspace& w = s->ws;
  const size_t logit_floats = (size_t)n * V;
  if (logit_floats > w.part_floats) return SP_E_CAPACITY;
  hipStream_t st = (hipStream_t)stream;
  hipError_t e = sp_launch_row_norm(c.dtype, x_root, head->norm, w.xn, n, d, c.rms_eps, st);
  if (e != hipSuccess) return hip_fail(s, e);
  ProfScope p(s, SP_K_VERIFY_HEAD, st);
  if (s->fast && V % 64 == 0 && d % 128 == 0) {
    int S = 1;
    e = sp_launch_gemm_bf16((const bf16_t*)w.xn, (const bf16_t*)head->wvocab, s->packed, w.part, n, V, d, 1,
                            logit_floats, &S, st);
  } else {
    e = sp_launch_gemm_simple(c.dtype, w.xn, head->wvocab, w.part, n, V, d, st);
  }
  if (e == hipSuccess)
    e = sp_launch_verify_sample(s->d_meta, s->d_tables, w.part, n, req_ids, V, temperature, top_p, top_k, u, result_dev, st);
  if (e == hipSuccess && result_host)
    e = hipMemcpyAsync(result_host, result_dev, sizeof(int32_t) * 2 * n, hipMemcpyDeviceToHost, st);
  return e == hipSuccess ? SP_OK : hip_fail(s, e);
}

int sp_tree_expand(sp_stage* s, int32_t req, int32_t n_bottom, const int32_t* bottom_nodes, int32_t k,
                   const int32_t* cand_tokens, const float* cand_probs, int32_t w, int32_t* out_parents,
                   int32_t* out_tokens, float* out_probs, int32_t* out_count, sp_stream stream) {
  if (!s || !bottom_nodes || !cand_tokens || !cand_probs || !out_parents || !out_tokens || !out_probs || !out_count)
    return SP_E_INVALID;
  HostReq* r = get_req(s, req);
  if (!r) return SP_E_BAD_REQ;
  if (r->pending) return SP_E_PENDING;
  if (n_bottom < 1 || n_bottom > SP_T || k < 1 || w < 0) return SP_E_INVALID;
  if ((long long)n_bottom * k > SP_EXPAND_MAX || w > SP_T) return SP_E_CAPACITY;
  ExpandArgs a;
  a.req = req; a.n_bottom = n_bottom; a.k = k; a.w = w;
  for (int i = 0; i < n_bottom; ++i) {
    const int b = bottom_nodes[i];
    // -1 (the root) only alone; otherwise live nodes in ascending order
    if (b == -1 ? n_bottom != 1 : (b < 0 || b >= r->T)) return SP_E_BAD_NODE;
    if (i > 0 && b <= bottom_nodes[i - 1]) return SP_E_INVALID;
    a.bottom[i] = (short)b;
  }
  hipError_t e = sp_launch_tree_expand(s->d_tables, a, cand_tokens, cand_probs, out_parents, out_tokens, out_probs,
                                       out_count, (hipStream_t)stream);
  return e == hipSuccess ? SP_OK : hip_fail(s, e);
}

int sp_tree_match(sp_stage* s, int32_t n, const int32_t* req_ids, int32_t* nodes_dev, int32_t* nodes_host,
                  sp_stream stream) {
  if (!s || !req_ids || !nodes_dev) return SP_E_INVALID;
  if (n < 0 || n > SP_MAX_BATCH_REQ) return SP_E_CAPACITY;
  for (int i = 0; i < n; ++i) {
    HostReq* r = get_req(s, req_ids[i]);
    if (!r) return SP_E_BAD_REQ;
    if (r->pending) return SP_E_PENDING;
  }
  if (n == 0) return SP_OK;
  hipStream_t st = (hipStream_t)stream;
  hipError_t e = sp_launch_tree_match(s->d_meta, s->d_tables, n, req_ids, nodes_dev, st);
  if (e == hipSuccess && nodes_host)
    e = hipMemcpyAsync(nodes_host, nodes_dev, sizeof(int32_t) * n, hipMemcpyDeviceToHost, st);
  return e == hipSuccess ? SP_OK : hip_fail(s, e);
}

int sp_profile_begin(sp_stage* s, int32_t kind, int32_t max_launches) {
  if (!s || kind <= SP_K_NONE || kind >= SP_K_KIND_COUNT || max_launches < 1) return SP_E_INVALID;
  while ((int)s->prof_ev.size() < 2 * max_launches) {
    hipEvent_t ev;
    hipError_t e = hipEventCreate(&ev);
    if (e != hipSuccess) return hip_fail(s, e);
    s->prof_ev.push_back(ev);
  }
  s->prof_kind = kind; s->prof_max = max_launches; s->prof_n = 0;
  s->prof_every = 1; s->prof_seen = 0; s->prof_group = 1;
  return SP_OK;
}

int sp_profile_sample_every(sp_stage* s, int32_t every) {
  if (!s || every < 1) return SP_E_INVALID;
  s->prof_every = every;
  s->prof_seen = 0;
  return SP_OK;
}

int sp_profile_end(sp_stage* s, int32_t* n_launches, float* total_ms) {
  if (!s) return SP_E_INVALID;
  float tot = 0.f;
  for (int i = 0; i < s->prof_n; ++i) {
    hipError_t e = hipEventSynchronize(s->prof_ev[2 * i + 1]);
    if (e != hipSuccess) return hip_fail(s, e);
    float ms = 0.f;
    e = hipEventElapsedTime(&ms, s->prof_ev[2 * i], s->prof_ev[2 * i + 1]);
    if (e != hipSuccess) return hip_fail(s, e);
    tot += ms;
  }
  if (n_launches) *n_launches = s->prof_n;
  if (total_ms) *total_ms = tot;
  s->prof_kind = 0; s->prof_n = 0;
  return SP_OK;
}

}  // extern "C"
