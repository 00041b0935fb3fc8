// Host-side Dynamic SplitFuse composer and KV block allocator.
//
// One decision per forward pass (paper Sec. 2.2).  Prompts are cut into chunks over
// several passes, only the chunk that ends the prompt generates (Sec. 3.2 rule 1), and
// chunks are fused with the running generations so the pass carries exactly the token
// budget when enough tokens wait (rule 2).  Generations go first so prompts never stall
// them.  Cache storage is handed out in fixed-size blocks (Sec. 2.1).
//
// Two more composition policies exist for comparison runs of the scheduling simulator: they
// are the behaviours the paper contrasts Dynamic SplitFuse with (Sec. 2.2, Sec. 3, Sec. 4.4),
// reduced to their batch decision:
//   prompt-first       whenever prompts wait, the pass processes whole prompts only (first
//                      come first served, as many as fit the token budget, the first one
//                      even if it is longer) and running generations wait; otherwise all
//                      generations run
//   whole-prompt-joins continuous batching with a bound on sequences only: every pass runs
//                      the generations and lets waiting prompts join whole, unsplit
// Neither splits a prompt; both use the same block allocator and rotation.
//
// When the pool runs dry the paper is silent.  By default a pass in which nothing can be
// scheduled is reported as FSF_ERR_NO_BLOCKS.  With FSF_EXHAUST_PREEMPT_NEWEST the sequence
// that arrived last among those holding blocks gives them back and starts over as a prompt of
// the tokens it had processed plus the generated token it was about to feed (its emitted
// tokens stay emitted), and the decision is taken again; the oldest sequence therefore always
// makes progress, and only a sequence that alone exceeds the pool still ends in
// FSF_ERR_NO_BLOCKS.
//
// Pure host code: no HIP calls.  Sequences live in a slab indexed by small integers;
// the two queues hold slab indices.  compose() works in two phases, plan then apply, so
// an error leaves the scheduler untouched.
#include <cstdint>
#include <deque>
#include <new>
#include <vector>

#include "fsf.h"

namespace {

struct Seq {
  int32_t seq_id = 0;
  int32_t prompt_len = 0;
  int32_t max_new = 0;
  int32_t n_cached = 0;
  int32_t emitted = 0;
  int64_t arrival = 0;  // order of fsf_sched_add_request calls
  bool live = false;
  std::vector<int32_t> blocks;
};

struct Planned {
  int32_t slot;   // slab index
  int32_t n_new;
  int32_t n_alloc;  // blocks to pop for this entry
  bool emits;
  bool is_decode;
};

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

}  // namespace

struct fsf_sched {
  int32_t token_budget;
  int32_t max_seqs;
  int32_t block_size;
  int64_t num_blocks;
  std::deque<int32_t> free_blocks;
  std::vector<Seq> slab;
  std::vector<int32_t> free_slots;
  std::deque<int32_t> prompts;   // slab indices, arrival order
  std::vector<int32_t> decodes;  // slab indices, rotation order
  std::vector<Planned> pending;
  bool has_pending = false;
  int32_t policy = FSF_POLICY_SPLITFUSE;
  int32_t exhaustion = FSF_EXHAUST_STALL;
  int64_t n_arrived = 0;
  int64_t n_preemptions = 0;
  int64_t tokens_discarded = 0;
};

namespace {

// FSF_EXHAUST_PREEMPT_NEWEST: take the blocks of the newest sequence that holds any.  False
// if fewer than two sequences hold blocks (nothing to take from).
bool preempt_newest(fsf_sched* s) {
  int32_t victim = -1, holders = 0;
  bool victim_decodes = false;
  auto look = [&](int32_t slot, bool is_decode) {
    const Seq& q = s->slab[slot];
    if (q.blocks.empty()) return;
    ++holders;
    if (victim < 0 || q.arrival > s->slab[victim].arrival) {
      victim = slot;
      victim_decodes = is_decode;
    }
  };
  for (int32_t slot : s->prompts) look(slot, false);
  for (int32_t slot : s->decodes) look(slot, true);
  if (holders < 2) return false;
  Seq& q = s->slab[victim];
  ++s->n_preemptions;
  s->tokens_discarded += q.n_cached;
  for (int32_t b : q.blocks) s->free_blocks.push_back(b);
  q.blocks.clear();
  if (victim_decodes) {
    for (auto it = s->decodes.begin(); it != s->decodes.end(); ++it)
      if (*it == victim) {
        s->decodes.erase(it);
        break;
      }
    q.prompt_len = q.n_cached + 1;
    auto pos = s->prompts.begin();
    while (pos != s->prompts.end() && s->slab[*pos].arrival < q.arrival) ++pos;
    s->prompts.insert(pos, victim);
  }
  q.n_cached = 0;
  return true;
}

}  // namespace

extern "C" int fsf_sched_create(fsf_sched** out, int32_t token_budget, int32_t max_seqs,
                                int32_t block_size, int64_t num_blocks,
                                const int32_t* free_list_order) {
  if (!out || token_budget < 1 || max_seqs < 1 || block_size < 1 || num_blocks < 1 ||
      num_blocks > INT32_MAX)
    return FSF_ERR_INVALID_ARG;
  if (free_list_order) {  // must be a permutation of 0..num_blocks-1
    std::vector<char> seen(static_cast<size_t>(num_blocks), 0);
    for (int64_t i = 0; i < num_blocks; ++i) {
      int32_t b = free_list_order[i];
      if (b < 0 || b >= num_blocks || seen[b]) return FSF_ERR_INVALID_ARG;
      seen[b] = 1;
    }
  }
  fsf_sched* s = new (std::nothrow) fsf_sched();
  if (!s) return FSF_ERR_INVALID_ARG;
  s->token_budget = token_budget;
  s->max_seqs = max_seqs;
  s->block_size = block_size;
  s->num_blocks = num_blocks;
  for (int64_t i = 0; i < num_blocks; ++i)
    s->free_blocks.push_back(free_list_order ? free_list_order[i] : static_cast<int32_t>(i));
  *out = s;
  return FSF_OK;
}

extern "C" void fsf_sched_destroy(fsf_sched* s) { delete s; }

extern "C" int fsf_sched_set_policy(fsf_sched* s, int32_t policy) {
  if (!s || policy < FSF_POLICY_SPLITFUSE || policy > FSF_POLICY_WHOLE_PROMPT_JOINS) return FSF_ERR_INVALID_ARG;
  if (s->has_pending || !s->prompts.empty() || !s->decodes.empty()) return FSF_ERR_INVALID_ARG;
  s->policy = policy;
  return FSF_OK;
}

extern "C" int fsf_sched_set_exhaustion(fsf_sched* s, int32_t mode) {
  if (!s || (mode != FSF_EXHAUST_STALL && mode != FSF_EXHAUST_PREEMPT_NEWEST)) return FSF_ERR_INVALID_ARG;
  if (s->has_pending || !s->prompts.empty() || !s->decodes.empty()) return FSF_ERR_INVALID_ARG;
  s->exhaustion = mode;
  return FSF_OK;
}

extern "C" int fsf_sched_preemptions(const fsf_sched* s, int64_t* n_preemptions_out, int64_t* tokens_discarded_out) {
  if (!s || !n_preemptions_out || !tokens_discarded_out) return FSF_ERR_INVALID_ARG;
  *n_preemptions_out = s->n_preemptions;
  *tokens_discarded_out = s->tokens_discarded;
  return FSF_OK;
}

extern "C" int fsf_sched_add_request(fsf_sched* s, int32_t seq_id, int32_t prompt_len,
                                     int32_t max_new_tokens) {
  if (!s || prompt_len < 1 || max_new_tokens < 1) return FSF_ERR_INVALID_ARG;
  int32_t slot;
  if (!s->free_slots.empty()) {
    slot = s->free_slots.back();
    s->free_slots.pop_back();
  } else {
    slot = static_cast<int32_t>(s->slab.size());
    s->slab.emplace_back();
  }
  Seq& q = s->slab[slot];
  q.seq_id = seq_id;
  q.prompt_len = prompt_len;
  q.max_new = max_new_tokens;
  q.n_cached = 0;
  q.emitted = 0;
  q.arrival = s->n_arrived++;
  q.live = true;
  q.blocks.clear();
  s->prompts.push_back(slot);
  return FSF_OK;
}

extern "C" int fsf_compose_batch(fsf_sched* s, fsf_seq_desc* descs_out, int32_t* block_tables_out,
                                 int32_t max_blocks, int32_t* n_seqs_out, int32_t* n_tokens_out,
                                 int32_t* emits_token_out) {
  if (!s || !descs_out || !block_tables_out || !n_seqs_out || !n_tokens_out || !emits_token_out ||
      max_blocks < 1)
    return FSF_ERR_INVALID_ARG;
  if (s->has_pending) return FSF_ERR_INVALID_ARG;

  const int64_t B = s->block_size;
  std::vector<Planned> plan;
  for (;;) {  // taken again after every preemption
  plan.clear();
  int64_t free_left = static_cast<int64_t>(s->free_blocks.size());
  int32_t budget_left = s->token_budget;
  int32_t seqs_left = s->max_seqs;

  // ---- the comparison policies never split a prompt
  bool prompt_pass = false;
  if (s->policy != FSF_POLICY_SPLITFUSE) {
    const bool prompt_first = s->policy == FSF_POLICY_PROMPT_FIRST;
    if (!prompt_first) {  // whole-prompt-joins: generations run in every pass
      for (int32_t slot : s->decodes) {
        if (budget_left == 0 || seqs_left == 0) break;
        const Seq& q = s->slab[slot];
        int64_t need = ceil_div(q.n_cached + 1, B) - ceil_div(q.n_cached, B);
        if (need > free_left) continue;
        if (static_cast<int64_t>(q.blocks.size()) + need > max_blocks) return FSF_ERR_INVALID_ARG;
        plan.push_back({slot, 1, static_cast<int32_t>(need), true, true});
        free_left -= need;
        --budget_left;
        --seqs_left;
      }
    }
    int64_t prompt_tokens = 0;
    for (int32_t slot : s->prompts) {
      if (seqs_left == 0) break;
      const Seq& q = s->slab[slot];
      const int64_t want = q.prompt_len;  // n_cached is 0: prompts are never split
      // prompt-first fills a token budget with whole prompts (the first always goes);
      // whole-prompt-joins knows no token budget
      if (prompt_first && prompt_tokens > 0 && prompt_tokens + want > s->token_budget) break;
      const int64_t need = ceil_div(want, B);
      if (need > free_left) break;  // waits for blocks; no later prompt overtakes it
      if (need > max_blocks) return FSF_ERR_INVALID_ARG;
      plan.push_back({slot, static_cast<int32_t>(want), static_cast<int32_t>(need), true, false});
      free_left -= need;
      prompt_tokens += want;
      --seqs_left;
    }
    prompt_pass = prompt_first && prompt_tokens > 0;
  }
  // ---- plan: generations first, one token each, rotation order
  // (prompt-first: only in a pass without prompts; whole-prompt-joins: done above)
  if (s->policy == FSF_POLICY_SPLITFUSE || (s->policy == FSF_POLICY_PROMPT_FIRST && !prompt_pass))
  for (int32_t slot : s->decodes) {
    if (budget_left == 0 || seqs_left == 0) break;
    const Seq& q = s->slab[slot];
    int64_t need = ceil_div(q.n_cached + 1, B) - ceil_div(q.n_cached, B);
    if (need > free_left) continue;  // cannot get its block: sits this pass out
    if (static_cast<int64_t>(q.blocks.size()) + need > max_blocks) return FSF_ERR_INVALID_ARG;
    plan.push_back({slot, 1, static_cast<int32_t>(need), true, true});
    free_left -= need;
    --budget_left;
    --seqs_left;
  }
  // ---- plan: prompt tokens fill the rest of the budget, first come first served
  if (s->policy == FSF_POLICY_SPLITFUSE)
  for (int32_t slot : s->prompts) {
    if (budget_left == 0 || seqs_left == 0) break;
    const Seq& q = s->slab[slot];
    int64_t want = q.prompt_len - q.n_cached;
    if (want > budget_left) want = budget_left;
    int64_t have = ceil_div(q.n_cached, B);
    int64_t room = (have + free_left) * B - q.n_cached;
    int64_t take = want < room ? want : room;
    if (take == 0) break;
    int64_t need = ceil_div(q.n_cached + take, B) - have;
    if (have + need > max_blocks) return FSF_ERR_INVALID_ARG;
    plan.push_back({slot, static_cast<int32_t>(take), static_cast<int32_t>(need),
                    q.n_cached + take == q.prompt_len, false});
    free_left -= need;
    budget_left -= static_cast<int32_t>(take);
    --seqs_left;
    if (take < want) break;  // blocks ran out: start no later prompt
  }

  if (!plan.empty() || (s->prompts.empty() && s->decodes.empty())) break;
  if (s->exhaustion != FSF_EXHAUST_PREEMPT_NEWEST || !preempt_newest(s)) {
    *n_seqs_out = 0;
    *n_tokens_out = 0;
    return FSF_ERR_NO_BLOCKS;
  }
  }  // for (;;)

  if (plan.empty()) {
    *n_seqs_out = 0;
    *n_tokens_out = 0;
    s->pending.clear();
    s->has_pending = true;  // an empty pass still pairs with step_done()
    return FSF_OK;
  }

  // ---- apply: pop blocks, write descriptors and tables
  int32_t q_off = 0;
  for (size_t k = 0; k < plan.size(); ++k) {
    Seq& q = s->slab[plan[k].slot];
    for (int32_t a = 0; a < plan[k].n_alloc; ++a) {
      q.blocks.push_back(s->free_blocks.front());
      s->free_blocks.pop_front();
    }
    descs_out[k].n_new = plan[k].n_new;
    descs_out[k].n_cached = q.n_cached;
    descs_out[k].q_offset = q_off;
    descs_out[k].seq_id = q.seq_id;
    emits_token_out[k] = plan[k].emits ? 1 : 0;
    int32_t* row = block_tables_out + static_cast<size_t>(k) * max_blocks;
    const int32_t nb = static_cast<int32_t>(q.blocks.size());
    for (int32_t b = 0; b < max_blocks; ++b) row[b] = b < nb ? q.blocks[b] : -1;
    q_off += plan[k].n_new;
  }
  *n_seqs_out = static_cast<int32_t>(plan.size());
  *n_tokens_out = q_off;
  s->pending.swap(plan);
  s->has_pending = true;
  return FSF_OK;
}

extern "C" int fsf_sched_step_done(fsf_sched* s) {
  if (!s || !s->has_pending) return FSF_ERR_INVALID_ARG;
  s->has_pending = false;

  // rotation: generations that ran move behind those that did not
  std::vector<char> ran(s->slab.size(), 0);
  for (const Planned& p : s->pending)
    if (p.is_decode) ran[p.slot] = 1;
  std::vector<int32_t> next;
  next.reserve(s->decodes.size() + s->pending.size());
  for (int32_t slot : s->decodes)
    if (!ran[slot]) next.push_back(slot);
  for (const Planned& p : s->pending)
    if (p.is_decode) next.push_back(p.slot);

  auto retire = [&](int32_t slot) {
    Seq& q = s->slab[slot];
    for (int32_t b : q.blocks) s->free_blocks.push_back(b);
    q.blocks.clear();
    q.live = false;
    s->free_slots.push_back(slot);
  };

  std::vector<char> gone(s->slab.size(), 0);
  for (const Planned& p : s->pending) {
    Seq& q = s->slab[p.slot];
    q.n_cached += p.n_new;
    if (p.emits) ++q.emitted;
    if (p.is_decode) {
      if (q.emitted == q.max_new) {
        gone[p.slot] = 1;
        retire(p.slot);
      }
    } else if (q.n_cached == q.prompt_len) {
      for (auto it = s->prompts.begin(); it != s->prompts.end(); ++it)
        if (*it == p.slot) {
          s->prompts.erase(it);
          break;
        }
      if (q.emitted == q.max_new)
        retire(p.slot);
      else
        next.push_back(p.slot);
    }
  }
  s->decodes.clear();
  for (int32_t slot : next)
    if (!gone[slot]) s->decodes.push_back(slot);
  s->pending.clear();
  return FSF_OK;
}

extern "C" int64_t fsf_sched_free_blocks(const fsf_sched* s) {
  return s ? static_cast<int64_t>(s->free_blocks.size()) : -1;
}

extern "C" int32_t fsf_sched_live_seqs(const fsf_sched* s) {
  return s ? static_cast<int32_t>(s->prompts.size() + s->decodes.size()) : -1;
}
