// Host-side exerciser for libfsf's CPU code, built with AddressSanitizer and
// UndefinedBehaviorSanitizer (python -m paper_2401_08671_amd.build --sanitize) and run by
// tests/test_sanitized_host.py.  It drives, without a GPU:
//   - the Dynamic SplitFuse composer and block allocator (fsf_sched_*, fsf_compose_batch) on a
//     request script read from stdin, printing every pass so that the test can compare the
//     schedules with the oracle composer's,
//   - the host-side planning of the attention call on the composed passes: workspace sizing
//     with several tunings, the cutting of prompt-chunk tiles (fsf_plan_prefill_groups), the
//     pass validation (fsf_validate_pass) on sound and on corrupted tables.
// Any sanitizer report ends the program with a non-zero status.
//
// stdin:  budget max_seqs block_size num_blocks max_blocks policy exhaustion n_requests
//         then n_requests lines: arrival_pass seq_id prompt_len max_new_tokens
// stdout: per pass "P n_seqs n_tokens" then per sequence "S seq_id n_new n_cached emits blocks...",
//         finally "E passes free_blocks preemptions"
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "fsf.h"
#include "fsf_measure.h"

static void die(const char* what, int st) {
  std::fprintf(stderr, "host_check: %s failed with %d (%s)\n", what, st, fsf_strerror(st));
  std::exit(3);
}

int main() {
  int budget, max_seqs, B, max_blocks, policy, exhaustion, n_req;
  long long num_blocks;
  if (std::scanf("%d %d %d %lld %d %d %d %d", &budget, &max_seqs, &B, &num_blocks, &max_blocks, &policy, &exhaustion, &n_req) != 8)
    return 2;
  struct Req { int pass, id, plen, gen; };
  std::vector<Req> reqs(n_req);
  for (auto& r : reqs)
    if (std::scanf("%d %d %d %d", &r.pass, &r.id, &r.plen, &r.gen) != 4) return 2;

  fsf_sched* s = nullptr;
  int st = fsf_sched_create(&s, budget, max_seqs, B, num_blocks, nullptr);
  if (st != FSF_OK) die("fsf_sched_create", st);
  if ((st = fsf_sched_set_policy(s, policy)) != FSF_OK) die("fsf_sched_set_policy", st);
  if ((st = fsf_sched_set_exhaustion(s, exhaustion)) != FSF_OK) die("fsf_sched_set_exhaustion", st);

  std::vector<fsf_seq_desc> descs(max_seqs);
  std::vector<int32_t> tables((size_t)max_seqs * max_blocks), emits(max_seqs), groups(4 * 4096);
  size_t next = 0;
  int pass = 0;
  for (;; ++pass) {
    while (next < reqs.size() && reqs[next].pass <= pass) {
      if ((st = fsf_sched_add_request(s, reqs[next].id, reqs[next].plen, reqs[next].gen)) != FSF_OK) die("fsf_sched_add_request", st);
      ++next;
    }
    if (fsf_sched_live_seqs(s) == 0 && next == reqs.size()) break;
    int32_t n_seqs = 0, n_tokens = 0;
    st = fsf_compose_batch(s, descs.data(), tables.data(), max_blocks, &n_seqs, &n_tokens, emits.data());
    if (st == FSF_ERR_NO_BLOCKS) {
      std::printf("X %d\n", pass);
      break;
    }
    if (st != FSF_OK) die("fsf_compose_batch", st);
    std::printf("P %d %d\n", n_seqs, n_tokens);
    for (int i = 0; i < n_seqs; ++i) {
      std::printf("S %d %d %d %d", descs[i].seq_id, descs[i].n_new, descs[i].n_cached, emits[i]);
      for (int b = 0; b < max_blocks && tables[(size_t)i * max_blocks + b] >= 0; ++b) std::printf(" %d", tables[(size_t)i * max_blocks + b]);
      std::printf("\n");
    }
    if (n_seqs > 0) {
      // the attention call's host side on this pass, for two head groupings and several tunings
      for (int variant = 0; variant < 4; ++variant) {
        fsf_tuning tn = {};
        tn.struct_bytes = (int32_t)sizeof(tn);
        tn.compute_units = variant == 1 ? 16 : 0;
        tn.decode_target_waves = variant == 2 ? 1 << 20 : 0;
        tn.decode_min_item_blocks = variant == 2 ? 1 : 0;
        tn.stream_chunk_slices = variant == 3 ? 16 : 0;
        tn.max_decode_items_extra = variant == 3 ? 64 : 0;
        fsf_attn_cfg cfg = {variant & 1 ? 32 : 8, variant & 1 ? 8 : 8, 128, B, variant == 2 ? 300 : 0, 0.088f, FSF_BF16, 0, num_blocks, &tn};
        int32_t bad_s = 0, bad_c = 0;
        if ((st = fsf_validate_pass(&cfg, descs.data(), tables.data(), n_seqs, max_blocks, n_tokens, &bad_s, &bad_c)) != FSF_OK)
          die("fsf_validate_pass on a composed pass", st);
        if (fsf_ragged_attention_workspace_bytes(&cfg, n_seqs, n_tokens, max_blocks) == 0) die("workspace_bytes", -1);
        const int32_t units = tn.compute_units ? tn.compute_units : 256;
        const int32_t n = fsf_plan_prefill_groups(&cfg, descs.data(), n_seqs, units, groups.data(), (int32_t)(groups.size() / 4));
        if (n < 0) die("fsf_plan_prefill_groups", n);
      }
      // a corrupted table must be reported, not read past
      const int32_t keep = tables[0];
      fsf_attn_cfg cfg = {8, 8, 128, B, 0, 0.088f, FSF_BF16, 0, num_blocks, nullptr};
      tables[0] = (int32_t)num_blocks;
      if (fsf_validate_pass(&cfg, descs.data(), tables.data(), n_seqs, max_blocks, n_tokens, nullptr, nullptr) != FSF_ERR_INVALID_ARG)
        die("fsf_validate_pass accepted a block id beyond the pool", 0);
      tables[0] = keep;
    }
    if ((st = fsf_sched_step_done(s)) != FSF_OK) die("fsf_sched_step_done", st);
    if (pass > 100000) die("too many passes", 0);
  }
  // the linear map's choice of tile shape and parts of k over a grid of shapes (host arithmetic only)
  for (int32_t m : {1, 31, 64, 65, 128, 129, 256, 257, 1024, 1025, 100000})
    for (int32_t n : {256, 5120, 27648, 1 << 20})
      for (int32_t k : {64, 512, 5120, 1 << 20}) {
        const size_t bytes = fsf_linear_workspace_bytes(m, n, k);
        if (bytes % 256 != 0 || bytes > (size_t)8 * m * n * sizeof(float) + 256) die("fsf_linear_workspace_bytes", (int)(bytes >> 20));
      }
  if (fsf_linear_workspace_bytes(0, 256, 64) != 0 || fsf_linear_workspace_bytes(1, 100, 64) != 0) die("fsf_linear_workspace_bytes on bad shapes", 0);
  long long n_pre = 0, tok = 0;
  fsf_sched_preemptions(s, (int64_t*)&n_pre, (int64_t*)&tok);
  std::printf("E %d %lld %lld\n", pass, (long long)fsf_sched_free_blocks(s), n_pre);
  fsf_sched_destroy(s);
  return 0;
}
