// Internal declarations shared by the translation units of the ADSA HIP library:
// launch plan (how the attended set is split over workgroups), workspace layout,
// and the kernel launchers the C-ABI layer calls.  Not part of the public ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "adsa.h"

namespace adsa {

constexpr int kWave = 64;
constexpr int kSelThreads = 256;       // select / compact-plan workgroup
constexpr int kMoveThreads = 256;
constexpr int kMaxChunks = 16;         // a list is split over at most this many workgroups

// Attend launch plan: a workgroup handles (sequence, head group, token chunk).
struct AttendPlan {
  int lanes_per_row;    // lanes that cover one (token, head) row with 16-byte loads
  bool head_major;      // [head][slot][D] cache: a wave-load takes consecutive tokens of ONE head
  int heads_per_group;  // heads one workgroup covers: 1 (head-major) or rows-per-wave-load (slot-major)
  int n_head_groups;    // ceil(n_heads / heads_per_group)
  int n_chunks;         // token chunks per sequence (grid.x); every sequence splits its own count evenly
  int chunk_max;        // upper bound of tokens in one chunk, + 1
  int waves;            // waves per attend workgroup: 4, 8 or 16
};

// Rows of adsa_seq.score: one accumulator per head for ATTN_MASS (the rank of a slot is their sum),
// a single row otherwise.
static inline int score_rows(const adsa_params& p) {
  if (p.score_mode == ADSA_SCORE_VCOS_FUSED) return 2 * p.n_heads;    // per head: |v|^2 share, v.u share
  return p.score_mode == ADSA_SCORE_ATTN_MASS ? p.n_heads : 1;
}
// Eq. 2-3 ranking in either form
static inline bool is_vcos(const adsa_params& p) {
  return p.score_mode == ADSA_SCORE_VCOS || p.score_mode == ADSA_SCORE_VCOS_FUSED;
}
constexpr int kVcosTags = 4;      // floats after u in adsa_seq.vcos_u: [0] 1 + step u belongs to, [1] 1 + step the score rows belong to

// Workspace layout (byte offsets from a 256-byte aligned base).
struct Workspace {
  size_t counters_off;     // int32 [n_seq][n_head_groups]  arrival counters (zero between launches)
  size_t persistent_bytes; // leading bytes that adsa_workspace_init zeroes and every launch leaves zero
  size_t logits_off;       // float [n_seq][n_heads][lg_stride]  scaled logits in log2 units
  size_t part_ml_off;      // float [n_seq][n_heads][n_chunks][2]   (m, l) per chunk
  size_t part_acc_off;     // float [n_seq][n_heads][n_chunks][head_dim]
  size_t plan_off;         // int32 [n_seq][4]   compaction: old n_res, first moved slot, did, new n_res
  size_t vcos_off;         // float [n_seq][cap]   inverse V norms of the candidates (0 = not a candidate)
  size_t vcos_u_off;       // float [n_seq][ceil(cap/64)][n_heads*head_dim]   per-tile partial sums of v^
  size_t vcos_s_off;       // float [n_seq][cap]   Eq. 3's S_i of the two-pass computation when score[] holds
                           //                      the fused form's rows (ADSA_SCORE_VCOS_FUSED)
  size_t total;
  int lg_stride;           // sel_cap rounded up to a multiple of 4
};

AttendPlan make_attend_plan(const adsa_params& p);
Workspace make_workspace(const adsa_params& p, const AttendPlan& plan);

static inline int elem_bytes(const adsa_params& p) { return p.dtype == ADSA_F32 ? 4 : 2; }

// Kernel launchers (each returns hipGetLastError() of its launch).
hipError_t launch_workspace_init(char* ws, const Workspace& w, hipStream_t st);
hipError_t launch_select(const adsa_params& p, adsa_seq* seqs, int32_t* sel_idx, int32_t* sel_cnt,
                         bool plan_append, hipStream_t st);
hipError_t launch_vcos(const adsa_params& p, adsa_seq* seqs, bool for_compaction, char* ws,
                       const Workspace& w, hipStream_t st);
int vcos_tiles(int cap);
// ADSA_SCORE_VCOS_FUSED, after the eviction plan: u <- u - evicted row + the row that turns candidate next step
// (or a fresh sum when u does not belong to this step)
hipError_t launch_vcos_advance(const adsa_params& p, adsa_seq* seqs, hipStream_t st);
size_t vcos_advance_lds_bytes(const adsa_params& p);
hipError_t launch_attend(const adsa_params& p, const AttendPlan& plan, adsa_seq* seqs, const void* q,
                         const void* k_new, const void* v_new, const int32_t* sel_idx, const int32_t* sel_cnt,
                         void* out, float* lse, char* ws, const Workspace& w, bool accumulate, bool append,
                         bool advance, bool new_f32, hipStream_t st, hipEvent_t ev_start, hipEvent_t ev_stop);
// grouped-query path (q_per_kv >= 2): matrix-core kernel, one workgroup per (sequence, cache head, chunk of the list)
constexpr size_t kGqaMaxLds = 128 * 1024;     // dynamic LDS one workgroup may ask for
int gqa_logit_stride(const adsa_params& p, int n_chunks);
int gqa_global_logit_stride(const adsa_params& p);
size_t gqa_lds_bytes(const adsa_params& p, int waves, int n_chunks);
hipError_t launch_attend_gqa(const adsa_params& p, const AttendPlan& plan, adsa_seq* seqs, const void* q,
                             const void* k_new, const void* v_new, const int32_t* sel_idx,
                             const int32_t* sel_cnt, void* out, float* lse, char* ws, const Workspace& w,
                             bool accumulate, bool append, bool advance, bool new_f32, hipStream_t st,
                             hipEvent_t ev_start, hipEvent_t ev_stop);
hipError_t launch_compact(const adsa_params& p, adsa_seq* seqs, int32_t* keep_map, char* ws,
                          const Workspace& w, bool advance_step, hipStream_t st);
// once per device, before the first launch there: kernels that may ask for more than 64 KB of dynamic LDS
hipError_t gqa_prepare_kernels();
hipError_t vcos_prepare_kernels();

}  // namespace adsa
