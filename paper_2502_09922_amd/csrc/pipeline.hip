// Execution pipeline over several stages of one model (2D pipelining, Section 4.3 of the
// paper, Fig. 6a): host code only.  Every stage runs on its own stream; the only coupling
// between streams is a pair of events per (stage boundary, micro-batch): "produced" (stage
// s has written the hand-off buffer) and "consumed" (stage s+1 has finished reading it).
#include "../../include/ls_stage.h"
#include "kernels.hpp"

#include <new>
#include <vector>

struct ls_pipeline {
  std::vector<ls_stage*> stages;
  ls_cfg cfg;
  bool last_has_head;  // the last stage ends at the model's last layer and the model has a vocabulary
  // events of micro-batch slot m at boundary s (between stage s and s+1): [m][s]
  std::vector<std::vector<hipEvent_t>> produced, consumed;
  std::vector<std::vector<char>> consumed_valid;  // consumed[m][s] has been recorded
};

namespace {

ls_status fail(ls_status code, const char* msg) {
  ls::set_last_error("%s", msg);
  return code;
}

bool same_model(const ls_cfg& a, const ls_cfg& b) {
  return a.dtype == b.dtype && a.n_layers_total == b.n_layers_total && a.hidden == b.hidden &&
         a.n_q_heads == b.n_q_heads && a.n_kv_heads == b.n_kv_heads && a.head_dim == b.head_dim && a.ffn == b.ffn &&
         a.vocab == b.vocab;
}

void destroy_events(ls_pipeline* p) {
  for (auto& row : p->produced)
    for (auto e : row)
      if (e) (void)hipEventDestroy(e);
  for (auto& row : p->consumed)
    for (auto e : row)
      if (e) (void)hipEventDestroy(e);
  p->produced.clear();
  p->consumed.clear();
  p->consumed_valid.clear();
}

// make sure event slots exist for micro-batches 0..n-1
ls_status grow(ls_pipeline* p, int n) {
  const size_t nb = p->stages.size() - 1;
  while ((int)p->produced.size() < n) {
    std::vector<hipEvent_t> pr(nb, nullptr), co(nb, nullptr);
    bool ok = true;
    for (size_t s = 0; s < nb && ok; ++s)
      ok = hipEventCreateWithFlags(&pr[s], hipEventDisableTiming) == hipSuccess &&
           hipEventCreateWithFlags(&co[s], hipEventDisableTiming) == hipSuccess;
    if (!ok) {
      for (auto e : pr) if (e) (void)hipEventDestroy(e);
      for (auto e : co) if (e) (void)hipEventDestroy(e);
      return fail(LS_ERR_HIP, "ls_pipeline_run: hipEventCreate failed");
    }
    p->produced.push_back(pr);
    p->consumed.push_back(co);
    p->consumed_valid.push_back(std::vector<char>(nb, 0));
  }
  return LS_OK;
}

}  // namespace

extern "C" {

ls_status ls_pipeline_create(ls_stage* const* stages, int n_stages, ls_pipeline** out) {
  if (!stages || !out || n_stages < 1) return fail(LS_ERR_INVALID_ARG, "ls_pipeline_create: bad arguments");
  ls_cfg first{};
  int prev_hi = 0;
  for (int i = 0; i < n_stages; ++i) {
    ls_cfg c{};
    int lo = 0, hi = 0;
    if (!stages[i] || ls_stage_info(stages[i], &c, &lo, &hi) != LS_OK)
      return fail(LS_ERR_INVALID_ARG, "ls_pipeline_create: NULL stage");
    if (i == 0) first = c;
    else if (!same_model(first, c)) return fail(LS_ERR_INVALID_ARG, "ls_pipeline_create: stages of different models");
    else if (lo != prev_hi) return fail(LS_ERR_INVALID_ARG, "ls_pipeline_create: stage spans are not consecutive");
    prev_hi = hi;
  }
  ls_pipeline* p = new (std::nothrow) ls_pipeline();
  if (!p) return fail(LS_ERR_OOM, "ls_pipeline_create: host allocation failed");
  p->stages.assign(stages, stages + n_stages);
  p->cfg = first;
  p->last_has_head = first.vocab && prev_hi == (int)first.n_layers_total;
  *out = p;
  return LS_OK;
}

void ls_pipeline_destroy(ls_pipeline* p) {
  if (!p) return;
  destroy_events(p);
  delete p;
}

ls_status ls_pipeline_run(ls_pipeline* p, int phase, const ls_microbatch* mbs, int n_micro, void* const* hip_streams) {
  if (!p || !mbs || !hip_streams || n_micro < 1 || (phase != 0 && phase != 1))
    return fail(LS_ERR_INVALID_ARG, "ls_pipeline_run: bad arguments");
  const int ns = (int)p->stages.size();
  // everything the host can see is checked before the first enqueue
  for (int m = 0; m < n_micro; ++m) {
    const ls_microbatch& mb = mbs[m];
    if (!mb.in || !mb.kv || !mb.out || (ns > 1 && !mb.handoff))
      return fail(LS_ERR_INVALID_ARG, "ls_pipeline_run: NULL pointer in a micro-batch");
    for (int s = 0; s + 1 < ns; ++s)
      if (!mb.handoff[s]) return fail(LS_ERR_INVALID_ARG, "ls_pipeline_run: NULL hand-off buffer");
    for (int s = 0; s < ns; ++s) {
      if (!mb.kv[s].k || !mb.kv[s].v || !mb.kv[s].seq_lens)
        return fail(LS_ERR_INVALID_ARG, "ls_pipeline_run: NULL pointer inside an ls_kv");
      if (phase == 0 && !mb.cu_seqlens_dev) return fail(LS_ERR_INVALID_ARG, "ls_pipeline_run: NULL cu_seqlens");
      // the stage's own checks of shape and state (limits, cu_seqlens, blocks enqueued for load)
      const ls_status rc = phase == 0 ? ls_stage_check_prefill(p->stages[s], mb.cu_seqlens_host, mb.batch, mb.total_tokens)
                                      : ls_stage_check_decode(p->stages[s], mb.batch, mb.max_ctx);
      if (rc != LS_OK) return rc;
    }
    if (mb.logits_out && !p->last_has_head)
      return fail(LS_ERR_INVALID_ARG, "ls_pipeline_run: logits_out given but the last stage has no LM head");
  }
  ls_status rc = grow(p, n_micro);
  if (rc != LS_OK) return rc;

  for (int m = 0; m < n_micro; ++m) {
    const ls_microbatch& mb = mbs[m];
    for (int s = 0; s < ns; ++s) {
      hipStream_t st = (hipStream_t)hip_streams[s];
      const void* in = s == 0 ? mb.in : mb.handoff[s - 1];
      void* out = s == ns - 1 ? mb.out : mb.handoff[s];
      // the previous stage has produced this micro-batch
      if (s > 0 && hipStreamWaitEvent(st, p->produced[m][s - 1], 0) != hipSuccess)
        return fail(LS_ERR_HIP, "ls_pipeline_run: hipStreamWaitEvent failed");
      // the next stage has consumed what an earlier call left in the hand-off buffer
      if (s + 1 < ns && p->consumed_valid[m][s] && hipStreamWaitEvent(st, p->consumed[m][s], 0) != hipSuccess)
        return fail(LS_ERR_HIP, "ls_pipeline_run: hipStreamWaitEvent failed");
      float* lg = s == ns - 1 ? mb.logits_out : nullptr;
      rc = phase == 0 ? ls_stage_prefill(p->stages[s], in, mb.cu_seqlens_dev, mb.cu_seqlens_host, mb.batch,
                                         mb.total_tokens, &mb.kv[s], out, lg, st)
                      : ls_stage_decode(p->stages[s], in, mb.batch, mb.max_ctx, &mb.kv[s], out, lg, st);
      if (rc != LS_OK) return rc;
      if (s + 1 < ns && hipEventRecord(p->produced[m][s], st) != hipSuccess)
        return fail(LS_ERR_HIP, "ls_pipeline_run: hipEventRecord failed");
      if (s > 0) {
        if (hipEventRecord(p->consumed[m][s - 1], st) != hipSuccess)
          return fail(LS_ERR_HIP, "ls_pipeline_run: hipEventRecord failed");
        p->consumed_valid[m][s - 1] = 1;
      }
    }
  }
  return LS_OK;
}

}  // extern "C"
