// C ABI of the ADSA HIP library: host-side argument validation and launch ordering.
// Every entry point only enqueues kernels on the caller's stream.
#include <vector>

#include "adsa_internal.h"

namespace adsa {
namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int validate_resolved(const adsa_params* p) {
  if (!p) return ADSA_ERR_NULL;
  if (p->dtype != ADSA_F32 && p->dtype != ADSA_BF16) return ADSA_ERR_DTYPE;
  if (p->score_mode < ADSA_SCORE_ATTN_MASS || p->score_mode > ADSA_SCORE_VCOS_FUSED) return ADSA_ERR_DTYPE;
  if (p->n_seq < 1 || p->n_seq > 65535) return ADSA_ERR_SHAPE;
  if (p->n_heads < 1 || p->n_heads > 256) return ADSA_ERR_SHAPE;
  if (p->head_dim != 64 && p->head_dim != 128) return ADSA_ERR_SHAPE;
  if (p->grid_h < 1 || p->grid_w < 1 || (long long)p->grid_h * p->grid_w > (1 << 24)) return ADSA_ERR_SHAPE;
  if (p->win_rows_back < 0 || p->win_col_radius < 0) return ADSA_ERR_SHAPE;
  if (p->sel_groups != 1) return ADSA_ERR_UNSUPPORTED;     // (resolve_params has rewritten the per-head form)
  if (is_vcos(*p) && (long long)p->n_heads * p->head_dim > 8192) return ADSA_ERR_UNSUPPORTED;
  if (p->cap < 1 || p->cap > ADSA_MAX_CAP) return ADSA_ERR_CAPACITY;
  if (p->sel_cap < 1 || p->sel_cap > p->cap) return ADSA_ERR_CAPACITY;
  const long long eb = p->dtype == ADSA_F32 ? 4 : 2;
  if (p->kv_slot_stride < 1 || p->kv_head_stride < 1) return ADSA_ERR_SHAPE;
  if ((p->kv_slot_stride * eb) % 16 != 0 || (p->kv_head_stride * eb) % 16 != 0) return ADSA_ERR_ALIGN;
  // rows of different (slot, head) must not overlap: one of the two supported nestings
  const bool slot_major = p->kv_head_stride >= p->head_dim &&
                          p->kv_slot_stride >= (long long)p->n_heads * p->kv_head_stride;
  const bool head_major = p->kv_slot_stride >= p->head_dim &&
                          p->kv_head_stride >= (long long)p->cap * p->kv_slot_stride;
  if (!slot_major && !head_major) return ADSA_ERR_SHAPE;
  if (!(p->softmax_scale >= 0.0f)) return ADSA_ERR_SHAPE;
  if (p->win_recent_m < 0) return ADSA_ERR_SHAPE;
  if (p->evict_policy < ADSA_EVICT_ROW_END || p->evict_policy > ADSA_EVICT_REUSE_SLOT) return ADSA_ERR_DTYPE;
  if (p->evict_policy != ADSA_EVICT_ROW_END && p->win_recent_m == 0) return ADSA_ERR_UNSUPPORTED;
  if (p->q_per_kv < 0 || p->q_per_kv > 16) return ADSA_ERR_SHAPE;
  if (p->score_mode == ADSA_SCORE_VCOS_FUSED) {      // u lives in LDS four times; rows are per cache head
    if (p->evict_policy != ADSA_EVICT_REUSE_SLOT || !head_major || p->kv_slot_stride >= p->kv_head_stride ||
        p->q_per_kv > 1)
      return ADSA_ERR_UNSUPPORTED;
    if (vcos_advance_lds_bytes(*p) > 64 * 1024) return ADSA_ERR_UNSUPPORTED;
    // m = 1: the token that turns candidate next step is not resident yet when the running sum is advanced
    if (p->win_recent_m < 2) return ADSA_ERR_UNSUPPORTED;
  }
  if (p->q_per_kv > 1) {       // grouped queries run on the bf16 matrix cores, logits of one chunk of the list in LDS
    if (p->dtype != ADSA_BF16) return ADSA_ERR_UNSUPPORTED;
    const AttendPlan gp = make_attend_plan(*p);
    if (gqa_lds_bytes(*p, gp.waves, gp.n_chunks) > kGqaMaxLds) return ADSA_ERR_UNSUPPORTED;
    // the kernel reaches a head's rows with 32-bit byte offsets
    if ((long long)p->cap * p->kv_slot_stride * 2 >= (1ll << 32)) return ADSA_ERR_UNSUPPORTED;
  }
  return ADSA_OK;
}

// The parameters the kernels run with.  sel_groups == 1: the caller's own.  sel_groups == n_heads (one attended
// set, one eviction history per head; Eq. 4 does not say which): every (sequence, head) IS a sequence of one cache
// head -- the caller passes n_seq * n_heads records, record b * n_heads + h describing head h of sequence b (its K/V
// rows kv_slot_stride apart, its own pos / score / counters), and sel_idx, sel_cnt, keep_map carry one row per record;
// q, k_new, v_new, out, lse keep their [n_seq][heads][...] layout, which is the same memory as
// [n_seq * n_heads][1 (* q_per_kv)][...].
int resolve_params(const adsa_params* p, adsa_params* eff) {
  if (!p) return ADSA_ERR_NULL;
  *eff = *p;
  if (p->sel_groups != 1) {
    if (p->n_heads < 1 || p->sel_groups != p->n_heads) return ADSA_ERR_UNSUPPORTED;
    if (p->n_seq < 1 || (long long)p->n_seq * p->n_heads > 65535) return ADSA_ERR_SHAPE;
    if (p->cap < 1 || p->kv_slot_stride < 1 || p->kv_head_stride < 1) return ADSA_ERR_SHAPE;
    eff->n_seq = p->n_seq * p->n_heads;
    eff->n_heads = 1;
    eff->sel_groups = 1;
    // one head per record: its rows are kv_slot_stride apart, whatever the nesting of the caller's cache
    eff->kv_head_stride = (long long)p->cap * p->kv_slot_stride;
  }
  return validate_resolved(eff);
}

// Per-device set-up that must not sit next to a launch (it would end up inside captured graphs, and tools that
// intercept launches see it interleaved with them): done at the library's first call on a device.
bool g_device_ready[64] = {};
int ensure_device_ready() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return ADSA_ERR_LAUNCH;
  if (!g_device_ready[dev]) {
    if (gqa_prepare_kernels() != hipSuccess || vcos_prepare_kernels() != hipSuccess) return ADSA_ERR_LAUNCH;
    g_device_ready[dev] = true;
  }
  return ADSA_OK;
}

int check_workspace(const adsa_params* p, const void* ws, size_t bytes, AttendPlan* plan, Workspace* w) {
  *plan = make_attend_plan(*p);
  *w = make_workspace(*p, *plan);
  if (!ws) return ADSA_ERR_WORKSPACE;
  if ((reinterpret_cast<uintptr_t>(ws) & 255u) != 0) return ADSA_ERR_ALIGN;
  if (bytes < w->total) return ADSA_ERR_WORKSPACE;
  return ADSA_OK;
}

// ---- benchmark timing hook: HIP events around the attention kernel, on the caller's stream
struct Profile {
  bool on = false;
  std::vector<hipEvent_t> ev;      // pairs (start, stop)
  size_t used = 0;
};
Profile g_prof;

hipEvent_t prof_event() {
  if (g_prof.used == g_prof.ev.size()) {
    hipEvent_t e;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    g_prof.ev.push_back(e);
  }
  return g_prof.ev[g_prof.used++];
}

hipError_t timed_attend(const adsa_params& p, const AttendPlan& plan, adsa_seq* seqs, const void* q,
                        const void* k_new, const void* v_new, const int32_t* sel_idx, const int32_t* sel_cnt,
                        void* out, float* lse, char* ws, const Workspace& w, bool accumulate, bool append,
                        bool advance, bool new_f32, hipStream_t st) {
  hipEvent_t e0 = nullptr, e1 = nullptr;
  if (g_prof.on) {
    e0 = prof_event();
    e1 = prof_event();
    if (!e0 || !e1) e0 = e1 = nullptr;
  }
  return launch_attend(p, plan, seqs, q, k_new, v_new, sel_idx, sel_cnt, out, lse, ws, w, accumulate, append,
                       advance, new_f32 && p.dtype == ADSA_BF16, st, e0, e1);
}

// ---- built-in scratch of adsa_step_static: one array per GPU, held until the process ends.  In host code
// the array's NAME is only a handle for hipGetSymbolAddress: the address kernels and fills are given is the
// one that call returns, kept per device.
constexpr size_t kStaticScratchBytes = ADSA_STATIC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;
struct StaticScratch {
  char* ptr = nullptr;          // device address of `scratch` on this GPU
  size_t zero_bytes = 0;        // leading bytes (arrival counters) the last call's layout kept at zero; 0 = none yet
};
StaticScratch g_static[kMaxDevices];

}  // namespace
}  // namespace adsa

static __device__ __align__(256) unsigned char scratch[adsa::kStaticScratchBytes];

namespace adsa {
namespace {

// Device address of this GPU's scratch array (resolved once per device, with that device current).
int static_scratch(StaticScratch** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return ADSA_ERR_LAUNCH;
  StaticScratch& s = g_static[dev];
  if (!s.ptr) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return ADSA_ERR_LAUNCH;
    s.ptr = static_cast<char*>(ptr);
    s.zero_bytes = 0;
  }
  *out = &s;
  return ADSA_OK;
}

// One whole decode step (the body of adsa_step / adsa_step_static); ws is laid out as w.
int step_launches(const adsa_params* p, const AttendPlan& plan, const Workspace& w, adsa_seq* seqs, const void* q,
                  const void* k_new, const void* v_new, void* out, float* lse, int32_t* sel_idx, int32_t* sel_cnt,
                  int32_t* keep_map, uint32_t flags, char* ws, hipStream_t st) {
  const bool compact = !(flags & ADSA_FLAG_NO_COMPACT);
  const bool vcos = is_vcos(*p);
  const bool accumulate = p->score_mode == ADSA_SCORE_ATTN_MASS;
  const bool streaming = p->evict_policy != ADSA_EVICT_ROW_END;
  if (streaming && compact) {          // Section 4.2 as written: make room BEFORE the insertion
    if (vcos && launch_vcos(*p, seqs, true, ws, w, st) != hipSuccess) return ADSA_ERR_LAUNCH;
    if (launch_compact(*p, seqs, keep_map, ws, w, false, st) != hipSuccess) return ADSA_ERR_LAUNCH;
    if (p->score_mode == ADSA_SCORE_VCOS_FUSED && launch_vcos_advance(*p, seqs, st) != hipSuccess)
      return ADSA_ERR_LAUNCH;
  }
  if (vcos && !streaming && launch_vcos(*p, seqs, false, ws, w, st) != hipSuccess) return ADSA_ERR_LAUNCH;
  if (launch_select(*p, seqs, sel_idx, sel_cnt, true, st) != hipSuccess) return ADSA_ERR_LAUNCH;
  if (timed_attend(*p, plan, seqs, q, k_new, v_new, sel_idx, sel_cnt, out, lse, ws, w, accumulate, true,
                   !compact || streaming, (flags & ADSA_FLAG_NEW_F32) != 0, st) != hipSuccess)
    return ADSA_ERR_LAUNCH;
  if (compact && !streaming) {
    if (vcos && launch_vcos(*p, seqs, true, ws, w, st) != hipSuccess) return ADSA_ERR_LAUNCH;
    if (launch_compact(*p, seqs, keep_map, ws, w, true, st) != hipSuccess) return ADSA_ERR_LAUNCH;
  }
  return ADSA_OK;
}

int check_step_args(const adsa_params* p, const adsa_seq* seqs, const void* q, const void* k_new, const void* v_new,
                    const void* out, const float* lse, const int32_t* sel_idx, const int32_t* sel_cnt,
                    const int32_t* keep_map, uint32_t flags, adsa_params* eff) {
  int rc = resolve_params(p, eff);      // *eff: the parameters the kernels run with
  if (rc) return rc;
  const bool compact = !(flags & ADSA_FLAG_NO_COMPACT);
  if (!seqs || !q || !k_new || !v_new || !out || !lse || !sel_idx || !sel_cnt) return ADSA_ERR_NULL;
  if (compact && !keep_map) return ADSA_ERR_NULL;
  if (!aligned16(q) || !aligned16(out) || !aligned16(k_new) || !aligned16(v_new)) return ADSA_ERR_ALIGN;
  return ADSA_OK;
}

}  // namespace
}  // namespace adsa

using namespace adsa;

extern "C" {

int adsa_version(void) { return ADSA_VERSION; }

const char* adsa_strerror(int code) {
  switch (code) {
    case ADSA_OK: return "ok";
    case ADSA_ERR_NULL: return "required pointer is NULL";
    case ADSA_ERR_SHAPE: return "size or window parameter out of range";
    case ADSA_ERR_DTYPE: return "unknown dtype or score mode";
    case ADSA_ERR_ALIGN: return "pointer or stride not 16-byte aligned";
    case ADSA_ERR_CAPACITY: return "cap or sel_cap out of range";
    case ADSA_ERR_WORKSPACE: return "workspace missing or too small";
    case ADSA_ERR_LAUNCH: return "HIP launch failed";
    case ADSA_ERR_UNSUPPORTED: return "not implemented in this build";
    case ADSA_ERR_STATIC_SCRATCH: return "parameters need more scratch than adsa_step_static's built-in buffer holds";
    default: return "unknown error";
  }
}

size_t adsa_workspace_bytes(const adsa_params* p) {
  adsa_params eff;
  if (resolve_params(p, &eff) != ADSA_OK) return 0;
  p = &eff;
  AttendPlan plan = make_attend_plan(*p);
  return make_workspace(*p, plan).total;
}

int adsa_workspace_init(const adsa_params* p, void* workspace, size_t workspace_bytes, void* stream) {
  adsa_params eff;
  int rc = resolve_params(p, &eff);
  if (rc) return rc;
  p = &eff;
  AttendPlan plan; Workspace w;
  rc = check_workspace(p, workspace, workspace_bytes, &plan, &w);
  if (rc) return rc;
  rc = ensure_device_ready();
  if (rc) return rc;
  if (launch_workspace_init((char*)workspace, w, reinterpret_cast<hipStream_t>(stream)) != hipSuccess)
    return ADSA_ERR_LAUNCH;
  return ADSA_OK;
}

int adsa_select(const adsa_params* p, adsa_seq* seqs, int32_t* sel_idx, int32_t* sel_cnt,
                uint32_t flags, void* workspace, size_t workspace_bytes, void* stream) {
  adsa_params eff;
  int rc = resolve_params(p, &eff);
  if (rc) return rc;
  p = &eff;
  if (!seqs || !sel_idx || !sel_cnt) return ADSA_ERR_NULL;
  rc = ensure_device_ready();
  if (rc) return rc;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  // (with the evict-one-when-full policies everything resident is attended: nothing to rank at selection time)
  if (p->score_mode == ADSA_SCORE_VCOS && p->evict_policy == ADSA_EVICT_ROW_END) {
    AttendPlan plan; Workspace w;
    rc = check_workspace(p, workspace, workspace_bytes, &plan, &w);
    if (rc) return rc;
    if (launch_vcos(*p, seqs, false, (char*)workspace, w, st) != hipSuccess) return ADSA_ERR_LAUNCH;
  }
  if (launch_select(*p, seqs, sel_idx, sel_cnt, (flags & ADSA_FLAG_PLAN_APPEND) != 0, st) != hipSuccess)
    return ADSA_ERR_LAUNCH;
  return ADSA_OK;
}

int adsa_attend(const adsa_params* p, adsa_seq* seqs, const void* q, const void* k_new,
                const void* v_new, const int32_t* sel_idx, const int32_t* sel_cnt, void* out,
                float* lse, uint32_t flags, void* workspace, size_t workspace_bytes, void* stream) {
  adsa_params eff;
  int rc = resolve_params(p, &eff);
  if (rc) return rc;
  p = &eff;
  if (!seqs || !q || !sel_idx || !sel_cnt || !out || !lse) return ADSA_ERR_NULL;
  const bool append = (flags & ADSA_FLAG_APPEND) != 0;
  if (append && (!k_new || !v_new)) return ADSA_ERR_NULL;
  if (!aligned16(q) || !aligned16(out)) return ADSA_ERR_ALIGN;
  if (append && (!aligned16(k_new) || !aligned16(v_new))) return ADSA_ERR_ALIGN;
  AttendPlan plan; Workspace w;
  rc = check_workspace(p, workspace, workspace_bytes, &plan, &w);
  if (rc) return rc;
  rc = ensure_device_ready();
  if (rc) return rc;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  const bool accumulate = p->score_mode == ADSA_SCORE_ATTN_MASS && !(flags & ADSA_FLAG_NO_ACCUMULATE);
  if (timed_attend(*p, plan, seqs, q, k_new, v_new, sel_idx, sel_cnt, out, lse, (char*)workspace, w, accumulate,
                   append, (flags & ADSA_FLAG_ADVANCE) != 0, (flags & ADSA_FLAG_NEW_F32) != 0, st) != hipSuccess)
    return ADSA_ERR_LAUNCH;
  return ADSA_OK;
}

int adsa_compact(const adsa_params* p, adsa_seq* seqs, int32_t* keep_map, uint32_t flags,
                 void* workspace, size_t workspace_bytes, void* stream) {
  adsa_params eff;
  int rc = resolve_params(p, &eff);
  if (rc) return rc;
  p = &eff;
  if (!seqs || !keep_map) return ADSA_ERR_NULL;
  AttendPlan plan; Workspace w;
  rc = check_workspace(p, workspace, workspace_bytes, &plan, &w);
  if (rc) return rc;
  rc = ensure_device_ready();
  if (rc) return rc;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  if (is_vcos(*p) && launch_vcos(*p, seqs, true, (char*)workspace, w, st) != hipSuccess)
    return ADSA_ERR_LAUNCH;
  if (launch_compact(*p, seqs, keep_map, (char*)workspace, w, (flags & ADSA_FLAG_ADVANCE) != 0, st) != hipSuccess)
    return ADSA_ERR_LAUNCH;
  if (p->score_mode == ADSA_SCORE_VCOS_FUSED && launch_vcos_advance(*p, seqs, st) != hipSuccess)
    return ADSA_ERR_LAUNCH;
  return ADSA_OK;
}

int adsa_step(const adsa_params* p, adsa_seq* seqs, const void* q, const void* k_new,
              const void* v_new, void* out, float* lse, int32_t* sel_idx, int32_t* sel_cnt,
              int32_t* keep_map, uint32_t flags, void* workspace, size_t workspace_bytes,
              void* stream) {
  adsa_params eff;
  int rc = check_step_args(p, seqs, q, k_new, v_new, out, lse, sel_idx, sel_cnt, keep_map, flags, &eff);
  if (rc) return rc;
  p = &eff;
  AttendPlan plan; Workspace w;
  rc = check_workspace(p, workspace, workspace_bytes, &plan, &w);
  if (rc) return rc;
  rc = ensure_device_ready();
  if (rc) return rc;
  return step_launches(p, plan, w, seqs, q, k_new, v_new, out, lse, sel_idx, sel_cnt, keep_map, flags,
                       (char*)workspace, reinterpret_cast<hipStream_t>(stream));
}

int adsa_step_static(const adsa_params* p, adsa_seq* seqs, const void* q, const void* k_new,
                     const void* v_new, void* out, float* lse, int32_t* sel_idx, int32_t* sel_cnt,
                     int32_t* keep_map, uint32_t flags, void* stream) {
  adsa_params eff;
  int rc = check_step_args(p, seqs, q, k_new, v_new, out, lse, sel_idx, sel_cnt, keep_map, flags, &eff);
  if (rc) return rc;
  p = &eff;
  const AttendPlan plan = make_attend_plan(*p);
  const Workspace w = make_workspace(*p, plan);
  if (w.total > kStaticScratchBytes) return ADSA_ERR_STATIC_SCRATCH;
  StaticScratch* sc = nullptr;
  rc = static_scratch(&sc);
  if (rc) return rc;
  rc = ensure_device_ready();
  if (rc) return rc;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  // The array keeps the previous call's contents.  The arrival counters at its head must start at zero: every
  // launch leaves its own counters zero, so only a call whose counter region differs from the previous call's
  // (it may reach into bytes that call used for something else) clears it, with a fill kernel.
  if (sc->zero_bytes != w.persistent_bytes) {
    if (launch_workspace_init(sc->ptr, w, st) != hipSuccess) return ADSA_ERR_LAUNCH;
    sc->zero_bytes = w.persistent_bytes;
  }
  return step_launches(p, plan, w, seqs, q, k_new, v_new, out, lse, sel_idx, sel_cnt, keep_map, flags, sc->ptr, st);
}

int adsa_profile_enable(int on) {
  g_prof.on = on != 0;
  g_prof.used = 0;
  if (!on) {                    // switching the hook off gives its events back
    for (hipEvent_t e : g_prof.ev) (void)hipEventDestroy(e);
    g_prof.ev.clear();
  }
  return ADSA_OK;
}

int adsa_profile_read(int64_t* n_launches, double* total_ms) {
  if (!n_launches || !total_ms) return ADSA_ERR_NULL;
  double tot = 0.0;
  int64_t n = 0;
  for (size_t i = 0; i + 1 < g_prof.used; i += 2) {
    if (hipEventSynchronize(g_prof.ev[i + 1]) != hipSuccess) return ADSA_ERR_LAUNCH;
    float ms = 0.0f;
    if (hipEventElapsedTime(&ms, g_prof.ev[i], g_prof.ev[i + 1]) != hipSuccess) return ADSA_ERR_LAUNCH;
    tot += ms;
    ++n;
  }
  *n_launches = n;
  *total_ms = tot;
  g_prof.used = 0;
  return ADSA_OK;
}

}  // extern "C"
