// C-ABI entry points: argument validation, path selection, launches.
//
// The entry points follow the paper's statement of the problem: a pass is a list of
// (tokens now, tokens cached) per sequence (Sec. 2) over a blocked cache (Sec. 2.1).
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <atomic>
#include <mutex>
#include <utility>
#include <vector>

#include "fsf_internal.h"
#include "fsf_measure.h"

namespace {

using fsf::Pass;

bool cfg_ok(const fsf_attn_cfg* c) {
  if (!c) return false;
  if (c->n_q_heads < 1 || c->n_kv_heads < 1 || c->n_q_heads % c->n_kv_heads) return false;
  if (c->head_dim < 1 || c->block_size < 1 || c->window < 0 || c->num_blocks < 1) return false;
  if (c->dtype != FSF_F32 && c->dtype != FSF_BF16 && c->dtype != FSF_F16) return false;
  return true;
}

int elem_size(const fsf_attn_cfg* c) { return c->dtype == FSF_F32 ? 4 : 2; }

Pass make_pass(const fsf_attn_cfg* c, const fsf_seq_desc* descs_dev, const int32_t* bt_dev,
               int32_t n_seqs, int32_t max_blocks, int32_t n_tokens) {
  Pass p;
  p.n_q_heads = c->n_q_heads;
  p.n_kv_heads = c->n_kv_heads;
  p.group = c->n_q_heads / c->n_kv_heads;
  p.head_dim = c->head_dim;
  p.block_size = c->block_size;
  p.window = c->window;
  p.scale = c->scale;
  p.dtype = c->dtype;
  p.n_seqs = n_seqs;
  p.max_blocks = max_blocks;
  p.n_tokens = n_tokens;
  p.descs = descs_dev;
  p.block_tables = bt_dev;
  return p;
}

// Descriptors must tile [0, n_tokens) in order and fit the block table.
bool descs_ok(const fsf_attn_cfg* c, const fsf_seq_desc* h, int32_t n_seqs, int32_t max_blocks,
              int32_t n_tokens) {
  int64_t off = 0;
  for (int32_t s = 0; s < n_seqs; ++s) {
    if (h[s].n_new < 1 || h[s].n_cached < 0 || h[s].q_offset != off) return false;
    const int64_t total = (int64_t)h[s].n_new + h[s].n_cached;
    if ((total + c->block_size - 1) / c->block_size > max_blocks) return false;
    off += h[s].n_new;
  }
  return off == n_tokens;
}

// The matrix-core path takes 2-byte dtypes, head_dim 128, blocks of 16 * 2^k tokens (the 16
// keys a wave copies or loads at a time never straddle a block and find their block with a
// shift), up to 16 query heads per KV head, and a cache block (all heads) below 4 GiB (its
// byte offsets are formed in 32-bit scalar multiplies).
bool fast_path_ok(const fsf_attn_cfg* c) {
  return !(c->flags & FSF_FLAG_FORCE_GENERIC) && (c->dtype == FSF_BF16 || c->dtype == FSF_F16) &&
         c->head_dim == fsf::kHeadDim && c->block_size >= 16 &&
         (c->block_size & (c->block_size - 1)) == 0 &&
         (uint64_t)c->n_kv_heads * c->block_size * fsf::kHeadDim * 2 < (1ull << 32) &&
         c->n_q_heads / c->n_kv_heads <= 16 && c->scale > 0.f;
}

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// Workspace sections of the matrix-core path, in order.
struct WsLayout {
  size_t dec_item_start, pre_tile_start, dec_prow_start, dec_rec, pre_tile_seq, split_rows, part_ml, part_acc, pre_part, total;
  size_t items_cap, prow_cap;  // streaming items and partial-result rows the sections hold
};

// The caller's fsf_tuning with every default filled in.  Reads only the fields the caller's
// struct_bytes covers.
struct Tuning {
  int decode_target_waves, decode_min_item_blocks;
  bool min_item_blocks_given, target_waves_given, prefill_split;
  int decode_hold;  // 0: results stored as units finish; 1: held back, eight-wave workgroups; 2: held back, single-wave workgroups
  int compute_units;  // 0: ask the device (only when a launch needs it)
  int max_decode_items_extra, max_prefill_split_units;
  int stream_max_slices;  // chunks of at most this many slices take the streaming kernel (0: one-row sequences only)
  int overlap;            // 0: one kernel after the other; 1: prompt-chunk tiles beside the streaming kernel on the
                          // library's second stream, units from the cost model; >= 8: on exactly this many units
};

Tuning resolve_tuning(const fsf_attn_cfg* c) {
  fsf_tuning t = {};
  if (c->tuning && c->tuning->struct_bytes > 0)
    memcpy(&t, c->tuning, std::min<size_t>(sizeof(t), (size_t)c->tuning->struct_bytes));
  Tuning r;
  r.decode_target_waves = t.decode_target_waves > 0 ? t.decode_target_waves : 4096;
  r.min_item_blocks_given = t.decode_min_item_blocks > 0;
  r.target_waves_given = t.decode_target_waves > 0;
  // no item shorter than 16 blocks, or 1024 keys where blocks are smaller than 64 tokens
  r.decode_min_item_blocks = r.min_item_blocks_given ? t.decode_min_item_blocks
                                                     : (c->block_size < 64 ? std::max(1, 1024 / c->block_size) : 16);
  r.decode_hold = t.decode_hold < 0 ? 0 : (t.decode_hold == 2 ? 2 : 1);
  r.prefill_split = t.prefill_split >= 0;
  r.compute_units = t.compute_units > 0 ? t.compute_units : 0;
  r.max_decode_items_extra = t.max_decode_items_extra > 0 ? t.max_decode_items_extra : fsf::kMaxDecodeItemsExtra;
  r.max_prefill_split_units = t.max_prefill_split_units > 0 ? std::min(t.max_prefill_split_units, fsf::kMaxPrefillSplitUnits)
                                                            : fsf::kMaxPrefillSplitUnits;
  r.overlap = t.overlap >= 8 ? (t.overlap / 8) * 8 : (t.overlap > 0 ? 1 : 0);
  r.stream_max_slices = t.stream_chunk_slices > 0 ? std::min(t.stream_chunk_slices, fsf::kMaxStreamSlices)
                                                  : (t.stream_chunk_slices < 0 ? 0 : fsf::kDefaultStreamSlices);
  return r;
}

// Streaming items a pass is cut into beyond one per slice: about target_waves wave units in all.
int64_t decode_target_items(const fsf_attn_cfg* c, const Tuning& tn) {
  int64_t t = tn.decode_target_waves / c->n_kv_heads;
  if (t > tn.max_decode_items_extra) t = tn.max_decode_items_extra;
  return t;  // may be 0: no cuts
}

WsLayout ws_layout(const fsf_attn_cfg* c, const Tuning& tn, int32_t n_seqs, int32_t n_tokens) {
  WsLayout w;
  // every slice of every streaming sequence is an item (at most one per token), plus the cuts
  w.items_cap = (size_t)n_tokens + (size_t)n_seqs + (size_t)decode_target_items(c, tn);
  // Rows whose keys are cut hold one partial result per cut.  Generation rows alone need at most
  // twice the extra items; short chunks bring up to 16 rows per item, so room for 16 per extra
  // item is kept, but never more than twice the limit on extra items: the host coarsens the cuts
  // of a pass that would need more.
  w.prow_cap = std::min<size_t>((size_t)fsf::kStreamCols * decode_target_items(c, tn), 2 * (size_t)tn.max_decode_items_extra);
  const size_t tiles_cap = (size_t)n_seqs + (size_t)n_tokens / fsf::kPrefillTileM;
  size_t off = 0;
  w.dec_item_start = off;
  off += align256(((size_t)n_seqs + 1) * sizeof(int32_t));
  w.pre_tile_start = off;
  off += align256(((size_t)n_seqs + 1) * sizeof(int32_t));
  w.dec_prow_start = off;
  off += align256(((size_t)n_seqs + 1) * sizeof(int32_t));
  w.dec_rec = off;
  off += align256(w.items_cap * sizeof(fsf::UnitRec));
  w.pre_tile_seq = off;
  off += align256(tiles_cap * sizeof(int32_t));
  w.split_rows = off;
  off += align256(((size_t)n_tokens + 1) * 2 * sizeof(int32_t));
  w.part_ml = off;
  off += align256(w.prow_cap * c->n_q_heads * 2 * sizeof(float));
  w.part_acc = off;
  off += align256(w.prow_cap * c->n_q_heads * fsf::kHeadDim * sizeof(float));
  // partial results of split prompt-chunk tiles: at most kMaxPrefillSplitUnits (tile, head, part) workgroups
  const size_t split_units = std::min<size_t>(tn.max_prefill_split_units, tiles_cap * c->n_q_heads * 16);
  w.pre_part = off;
  off += align256(split_units * fsf::kPrefillTileM * fsf::kPrefillPartRowFloats * sizeof(float));
  w.total = off;
  return w;
}

int compute_units() { return fsf::device_compute_units(); }

// Which prompt-chunk tiles are cut along their keys (see PrefillSplit).  n_steps[t] = 64-key
// steps of tile t.  Workgroups (tile x head) take one compute unit each.
//   heavy: with an even spread every unit would work `even` steps; a tile with more steps than
//          that would run on after everything else has finished, so it is cut into parts of at
//          most `even` steps, or, when all workgroups fit one round anyway, into as many parts
//          as its share of the units (never shorter than kPrefillMinPartSteps); the
//          kMaxHeavyTiles longest such tiles are taken
//   tail:  when the last round of workgroups is at most half full, the tiles of that round are
//          cut into as many parts as fill the round
fsf::PrefillSplit plan_prefill_split(const std::vector<int>& n_steps, int H, int cus, bool allow,
                                     int max_split_units = fsf::kMaxPrefillSplitUnits) {
  fsf::PrefillSplit sp = {};
  const int n_tiles = (int)n_steps.size();
  if (!allow || n_tiles == 0) return sp;
  int64_t total = 0;
  for (int s : n_steps) total += s;
  const int64_t even = std::max<int64_t>((total * H + cus - 1) / cus, fsf::kPrefillMinPartSteps);
  int budget = max_split_units / H;  // (tile, part) groups with partial results
  const bool one_round = (int64_t)n_tiles * H <= cus;
  // ---- heavy tiles
  std::vector<int> order(n_tiles);
  for (int t = 0; t < n_tiles; ++t) order[t] = t;
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return n_steps[a] > n_steps[b]; });
  std::vector<std::pair<int, int>> heavy;  // (tile, parts)
  for (int t : order) {
    if ((int)heavy.size() == fsf::kMaxHeavyTiles || n_steps[t] <= even) break;
    // several rounds of workgroups: parts of at most the even share.  Less than one round: every
    // tile gets the share of the units that its steps are of all steps, rounded down, so that
    // the parts still fit one round
    int64_t want = one_round ? (int64_t)cus * n_steps[t] / (total * H) : (n_steps[t] + even - 1) / even;
    int parts = (int)std::min<int64_t>(want, 16);
    parts = std::min(parts, n_steps[t] / fsf::kPrefillMinPartSteps);
    parts = std::min(parts, budget);
    if (parts < 2) continue;
    heavy.push_back({t, parts});
    budget -= parts;
  }
  std::sort(heavy.begin(), heavy.end(), [](auto a, auto b) { return a.first > b.first; });  // descending tile index
  sp.n_heavy = (int)heavy.size();
  for (int k = 0; k < sp.n_heavy; ++k) {
    sp.heavy_tile[k] = heavy[k].first;
    sp.heavy_parts[k] = heavy[k].second;
  }
  // ---- tail tiles: all of the partial round (an unsplit workgroup left in it would last as long
  // as the round did before), whole tiles only
  const int64_t groups = fsf::prefill_groups(n_tiles, sp);
  const int64_t tail = groups * H % cus;
  const int n_plain = n_tiles - sp.n_heavy;
  if (tail == 0 || 2 * tail > cus || n_plain == 0 || groups * H < cus) return sp;
  const int tail_tiles = (int)std::min<int64_t>((tail + H - 1) / H, n_plain);
  int parts = std::max(2, (int)((cus + (int64_t)tail_tiles * H / 2) / ((int64_t)tail_tiles * H)));
  int min_steps = 1 << 30;
  sp.tail_tiles = tail_tiles;  // for prefill_nth_plain_tile below
  for (int a = 0; a < tail_tiles; ++a) min_steps = std::min(min_steps, n_steps[fsf::prefill_nth_plain_tile(a, sp)]);
  parts = std::min(std::min(parts, 16), min_steps / fsf::kPrefillMinPartSteps);
  parts = std::min(parts, budget / tail_tiles);
  if (parts < 2) {
    sp.tail_tiles = 0;
    return sp;
  }
  sp.tail_parts = parts;
  return sp;
}

// 64-key steps of every prompt-chunk tile of the pass, in tile order (sequence order, then rows)
std::vector<int> prefill_tile_steps_of(const fsf_attn_cfg* c, const Tuning& tn, const fsf_seq_desc* h, int32_t n_seqs) {
  std::vector<int> steps;
  for (int32_t s = 0; s < n_seqs; ++s) {
    if (fsf::is_streaming(h[s].n_new, c->n_q_heads / c->n_kv_heads, tn.stream_max_slices)) continue;
    for (int i0 = 0; i0 < h[s].n_new; i0 += fsf::kPrefillTileM)
      steps.push_back(fsf::prefill_tile_steps(h[s].n_cached, i0, std::min(i0 + fsf::kPrefillTileM, h[s].n_new),
                                              c->window));
  }
  return steps;
}

// one fused grid is launched only for blocks of 32 tokens or more, and never with split tiles
bool fused_launch(const fsf_attn_cfg* c) { return (c->flags & FSF_FLAG_FUSED_LAUNCH) && c->block_size >= 32; }

fsf::PrefillSplit choose_prefill_split(const fsf_attn_cfg* c, const Tuning& tn, const fsf_seq_desc* h, int32_t n_seqs) {
  const int cus = tn.compute_units ? tn.compute_units : compute_units();  // tests force splits with a small value
  const bool allow = !fused_launch(c) && tn.prefill_split;
  return plan_prefill_split(prefill_tile_steps_of(c, tn, h, n_seqs), c->n_q_heads, cus, allow, tn.max_prefill_split_units);
}

}  // namespace

extern "C" const char* fsf_strerror(int status) {
  switch (status) {
    case FSF_OK: return "ok";
    case FSF_ERR_INVALID_ARG: return "invalid argument";
    case FSF_ERR_UNSUPPORTED: return "unsupported dtype, head_dim or group size";
    case FSF_ERR_WORKSPACE: return "workspace missing or too small";
    case FSF_ERR_NO_BLOCKS: return "no free KV block";
    case FSF_ERR_HIP: return "HIP runtime error";
    default: return "unknown status";
  }
}

extern "C" int fsf_version(void) { return 100; }

extern "C" int32_t fsf_plan_prefill_groups(const fsf_attn_cfg* cfg, const fsf_seq_desc* descs_host,
                                           int32_t n_seqs, int32_t compute_units_assumed,
                                           int32_t* groups_out, int32_t cap) {
  if (!cfg_ok(cfg) || !descs_host || n_seqs < 0 || compute_units_assumed < 1 || (cap > 0 && !groups_out))
    return -1;
  const std::vector<int> steps = prefill_tile_steps_of(cfg, resolve_tuning(cfg), descs_host, n_seqs);
  const fsf::PrefillSplit sp = plan_prefill_split(steps, cfg->n_q_heads, compute_units_assumed, true);
  const int n = fsf::prefill_groups((int)steps.size(), sp);
  for (int g = 0; g < n && g < cap; ++g) {
    const fsf::PrefillWork w = fsf::prefill_group_to_work(g, (int)steps.size(), sp);
    groups_out[4 * g] = w.tile;
    groups_out[4 * g + 1] = w.part;
    groups_out[4 * g + 2] = w.n_parts;
    groups_out[4 * g + 3] = w.slab;
  }
  return n;
}

extern "C" int fsf_validate_pass(const fsf_attn_cfg* cfg, const fsf_seq_desc* descs_host,
                                 const int32_t* block_tables_host, int32_t n_seqs, int32_t max_blocks,
                                 int32_t n_tokens, int32_t* bad_seq_out, int32_t* bad_column_out) {
  auto bad = [&](int32_t s, int32_t col) {
    if (bad_seq_out) *bad_seq_out = s;
    if (bad_column_out) *bad_column_out = col;
    return (int)FSF_ERR_INVALID_ARG;
  };
  if (!cfg_ok(cfg) || n_seqs < 0 || n_tokens < 0 || max_blocks < 1) return bad(-1, -1);
  if (n_seqs == 0) return n_tokens == 0 ? (int)FSF_OK : bad(-1, -1);
  if (!descs_host || !block_tables_host) return bad(-1, -1);
  int64_t off = 0;
  for (int32_t s = 0; s < n_seqs; ++s) {  // descriptors tile [0, n_tokens) and fit the table
    const fsf_seq_desc& d = descs_host[s];
    const int64_t total = (int64_t)d.n_new + d.n_cached;
    if (d.n_new < 1 || d.n_cached < 0 || d.q_offset != off || (total + cfg->block_size - 1) / cfg->block_size > max_blocks)
      return bad(s, -1);
    off += d.n_new;
  }
  if (off != n_tokens) return bad(-1, -1);
  // every table entry the pass dereferences names a block of the pool, and none is named twice
  std::vector<bool> seen((size_t)cfg->num_blocks, false);
  for (int32_t s = 0; s < n_seqs; ++s) {
    const int64_t total = (int64_t)descs_host[s].n_new + descs_host[s].n_cached;
    const int32_t used = (int32_t)((total + cfg->block_size - 1) / cfg->block_size);
    for (int32_t b = 0; b < used; ++b) {
      const int32_t id = block_tables_host[(int64_t)s * max_blocks + b];
      if (id < 0 || id >= cfg->num_blocks || seen[(size_t)id]) return bad(s, b);
      seen[(size_t)id] = true;
    }
  }
  return FSF_OK;
}

extern "C" int fsf_kv_append(const fsf_attn_cfg* cfg, const void* k_new, const void* v_new,
                             void* k_cache, void* v_cache, const fsf_seq_desc* descs_dev,
                             const int32_t* block_tables_dev, int32_t n_seqs, int32_t max_blocks,
                             int32_t n_tokens, void* hip_stream) {
  if (!cfg_ok(cfg) || n_seqs < 0 || n_tokens < 0 || max_blocks < 1) return FSF_ERR_INVALID_ARG;
  if (n_seqs == 0 || n_tokens == 0) return FSF_OK;
  if (!k_new || !v_new || !k_cache || !v_cache || !descs_dev || !block_tables_dev)
    return FSF_ERR_INVALID_ARG;
  if ((cfg->head_dim * elem_size(cfg)) % 4) return FSF_ERR_UNSUPPORTED;
  if (((uintptr_t)k_new | (uintptr_t)v_new | (uintptr_t)k_cache | (uintptr_t)v_cache) & 3) return FSF_ERR_INVALID_ARG;
  const Pass p = make_pass(cfg, descs_dev, block_tables_dev, n_seqs, max_blocks, n_tokens);
  const hipError_t e =
      fsf::launch_kv_append(p, k_new, v_new, k_cache, v_cache, (hipStream_t)hip_stream);
  return e == hipSuccess ? FSF_OK : FSF_ERR_HIP;
}

extern "C" int fsf_kv_append_rotary(const fsf_attn_cfg* cfg, const void* k_new, const void* v_new,
                                    void* k_cache, void* v_cache, const fsf_seq_desc* descs_dev,
                                    const fsf_seq_desc* descs_host, const int32_t* block_tables_dev,
                                    int32_t n_seqs, int32_t max_blocks, int32_t n_tokens,
                                    const float* cos_sin_dev, int32_t table_positions, void* hip_stream) {
  if (!cfg_ok(cfg) || n_seqs < 0 || n_tokens < 0 || max_blocks < 1 || table_positions < 0)
    return FSF_ERR_INVALID_ARG;
  if (n_seqs == 0 || n_tokens == 0) return FSF_OK;
  if (!k_new || !v_new || !k_cache || !v_cache || !descs_dev || !descs_host || !block_tables_dev || !cos_sin_dev)
    return FSF_ERR_INVALID_ARG;
  if (cfg->head_dim % 2) return FSF_ERR_UNSUPPORTED;
  if (!descs_ok(cfg, descs_host, n_seqs, max_blocks, n_tokens)) return FSF_ERR_INVALID_ARG;
  for (int32_t s = 0; s < n_seqs; ++s)  // every position must have its row of angles
    if ((int64_t)descs_host[s].n_cached + descs_host[s].n_new > table_positions) return FSF_ERR_INVALID_ARG;
  const Pass p = make_pass(cfg, descs_dev, block_tables_dev, n_seqs, max_blocks, n_tokens);
  const hipError_t e = fsf::launch_kv_append_rotary(p, k_new, v_new, k_cache, v_cache, cos_sin_dev,
                                                    (hipStream_t)hip_stream);
  return e == hipSuccess ? FSF_OK : FSF_ERR_HIP;
}

extern "C" int fsf_rotary_q(const fsf_attn_cfg* cfg, void* q, const fsf_seq_desc* descs_dev,
                            const fsf_seq_desc* descs_host, int32_t n_seqs, int32_t n_tokens,
                            const float* cos_sin_dev, int32_t table_positions, void* hip_stream) {
  if (!cfg_ok(cfg) || n_seqs < 0 || n_tokens < 0 || table_positions < 0) return FSF_ERR_INVALID_ARG;
  if (n_seqs == 0 || n_tokens == 0) return FSF_OK;
  if (!q || !descs_dev || !descs_host || !cos_sin_dev) return FSF_ERR_INVALID_ARG;
  if (cfg->head_dim % 2) return FSF_ERR_UNSUPPORTED;
  if (!descs_ok(cfg, descs_host, n_seqs, INT32_MAX, n_tokens)) return FSF_ERR_INVALID_ARG;
  for (int32_t s = 0; s < n_seqs; ++s)
    if ((int64_t)descs_host[s].n_cached + descs_host[s].n_new > table_positions) return FSF_ERR_INVALID_ARG;
  const Pass p = make_pass(cfg, descs_dev, nullptr, n_seqs, 1, n_tokens);
  const hipError_t e = fsf::launch_rotary_q(p, q, cos_sin_dev, (hipStream_t)hip_stream);
  return e == hipSuccess ? FSF_OK : FSF_ERR_HIP;
}

namespace {

int linear_args_ok(int32_t dtype, const void* x, const void* w, const void* y, int32_t n_tokens, int32_t n_out,
                   int32_t k) {
  if (n_tokens < 0 || n_out < 1 || k < 1) return FSF_ERR_INVALID_ARG;
  if (dtype != FSF_BF16 && dtype != FSF_F16 && dtype != FSF_F32) return FSF_ERR_INVALID_ARG;
  if (n_tokens == 0) return FSF_OK;
  if (!x || !w || !y || (((uintptr_t)x | (uintptr_t)w | (uintptr_t)y) & 15)) return FSF_ERR_INVALID_ARG;
  // the kernel's tiling: 256 output features and 64 k-elements at a time, byte offsets in 31 bits
  if (dtype == FSF_F32 || n_out % 256 || k % 64 || (int64_t)n_tokens * k * 2 >= (1ll << 31) ||
      (int64_t)n_out * k * 2 >= (1ll << 31))
    return FSF_ERR_UNSUPPORTED;
  return FSF_OK;
}

}  // namespace

extern "C" int fsf_linear(int32_t dtype, const void* x, const void* w, void* y, int32_t n_tokens, int32_t n_out,
                          int32_t k, void* hip_stream) {
  const int st = linear_args_ok(dtype, x, w, y, n_tokens, n_out, k);
  if (st != FSF_OK || n_tokens == 0) return st;
  const hipError_t e = fsf::launch_linear(dtype, x, w, y, n_tokens, n_out, k, nullptr, 0, (hipStream_t)hip_stream);
  return e == hipSuccess ? FSF_OK : FSF_ERR_HIP;
}

extern "C" size_t fsf_linear_workspace_bytes(int32_t n_tokens, int32_t n_out, int32_t k) {
  if (n_tokens < 1 || n_out < 1 || k < 1 || n_out % 256 || k % 64) return 0;
  const int splits = fsf::linear_splits(n_tokens, n_out, k, compute_units(), ~(size_t)0);
  return splits > 1 ? align256((size_t)splits * n_tokens * n_out * sizeof(float)) : 0;
}

extern "C" int fsf_linear_ws(int32_t dtype, const void* x, const void* w, void* y, int32_t n_tokens, int32_t n_out,
                             int32_t k, void* workspace, size_t workspace_bytes, void* hip_stream) {
  const int st = linear_args_ok(dtype, x, w, y, n_tokens, n_out, k);
  if (st != FSF_OK || n_tokens == 0) return st;
  if (workspace && ((uintptr_t)workspace & 15)) return FSF_ERR_WORKSPACE;
  const hipError_t e = fsf::launch_linear(dtype, x, w, y, n_tokens, n_out, k, workspace, workspace ? workspace_bytes : 0,
                                          (hipStream_t)hip_stream);
  return e == hipSuccess ? FSF_OK : FSF_ERR_HIP;
}

extern "C" size_t fsf_ragged_attention_workspace_bytes(const fsf_attn_cfg* cfg, int32_t n_seqs,
                                                       int32_t n_tokens, int32_t max_blocks) {
  if (!cfg_ok(cfg) || n_seqs < 0 || n_tokens < 0 || max_blocks < 1) return 0;
  if (!fast_path_ok(cfg)) return 256;
  return ws_layout(cfg, resolve_tuning(cfg), n_seqs, n_tokens).total;
}

namespace {

// A second stream and two events per device, created on first use and kept until the process
// ends (host-side runtime objects; no device memory).  Default priority, like the caller's.
constexpr int kMaxOverlapUnits = 16;  // compute units the streaming kernel gives up without slowing down

constexpr int kSideEvents = 16;       // fork/join event pairs used in turn, so that a pair is not recorded again
                                      // while a pass a few calls back may still be waiting on it
struct SideStream {
  hipStream_t stream = nullptr;
  hipEvent_t fork[kSideEvents] = {}, join[kSideEvents] = {};
  unsigned next = 0;
  bool ok = false, tried = false;
};
SideStream g_side[64];
std::mutex g_side_mutex;

SideStream* side_stream() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
  std::lock_guard<std::mutex> lock(g_side_mutex);
  SideStream& s = g_side[dev];
  if (!s.tried) {
    s.tried = true;
    s.ok = hipStreamCreateWithFlags(&s.stream, hipStreamNonBlocking) == hipSuccess;
    for (int i = 0; i < kSideEvents && s.ok; ++i)
      s.ok = hipEventCreateWithFlags(&s.fork[i], hipEventDisableTiming) == hipSuccess &&
             hipEventCreateWithFlags(&s.join[i], hipEventDisableTiming) == hipSuccess;
  }
  return s.ok ? &s : nullptr;
}

// How many compute units the prompt-chunk tiles of a pass get when they run beside the streaming
// kernel, so that both finish at about the same time: their share of the pass's compute-unit
// time (a tile step, 64 keys x 256 rows of one head, takes about 1.7 us of a unit, the up to 8
// steps with masked scores 2 us more each, a workgroup 10 us more; the streaming kernel moves
// about 6.7 TB/s with all units).  0: the share is too
// large, run one kernel after the other.  Measured: the streaming kernel does not notice the
// loss of 8 or 16 units (it is bound by HBM, and the prompt-chunk work hides behind it entirely:
// the 2048- and 4096-token benchmark passes gain 3..6 %), but with a sixth of the units gone it
// slows down by as much (passes of the long-prompt stream whose chunk is most of the budget:
// 3 % slower than one after the other).
int overlap_units(const std::vector<int>& tile_steps, int n_q_heads, int64_t stream_bytes, int cus) {
  double pre_us = 0.0;
  for (int st : tile_steps) pre_us += (1.7 * st + 2.0 * std::min(st, 8) + 10.0) * n_q_heads;   // unit-microseconds
  const double dec_us = (double)stream_bytes / 6.7e6 * cus;           // unit-microseconds with all units
  if (pre_us <= 0.0 || dec_us <= 0.0) return 0;
  // Whole multiples of 8: workgroups are dealt to the chip's 8 dies in turn, so the streaming
  // kernel's grid then leaves the same number of units empty on every die.  (With an uneven
  // split some die is asked to hold one workgroup more than it has units; that workgroup starts
  // when another has finished, and the launch lasts up to twice as long.)
  const int units = std::max(8, (int)(cus * pre_us / (pre_us + dec_us) / 8.0 + 0.5) * 8);
  return units <= kMaxOverlapUnits ? units : 0;
}

}  // namespace

namespace {

// Checks shared by the two attention entry points; FSF_OK means there is work to launch.
int attention_args_ok(const fsf_attn_cfg* cfg, const void* q, const void* k_cache, const void* v_cache,
                      const fsf_seq_desc* descs_dev, const fsf_seq_desc* descs_host,
                      const int32_t* block_tables_dev, int32_t n_seqs, int32_t max_blocks, int32_t n_tokens,
                      const void* out) {
  if (!cfg_ok(cfg) || n_seqs < 0 || n_tokens < 0 || max_blocks < 1) return FSF_ERR_INVALID_ARG;
  if (!q || !k_cache || !v_cache || !descs_dev || !descs_host || !block_tables_dev || !out)
    return FSF_ERR_INVALID_ARG;
  if (!descs_ok(cfg, descs_host, n_seqs, max_blocks, n_tokens)) return FSF_ERR_INVALID_ARG;
  if (cfg->head_dim > 256) return FSF_ERR_UNSUPPORTED;
  return FSF_OK;
}

// The pass itself: arguments are valid, the workspace holds ws_layout(cfg, tn, ...).total bytes.
int run_attention(const fsf_attn_cfg* cfg, const Tuning& tn, const void* q, const void* k_cache,
                  const void* v_cache, const fsf_seq_desc* descs_dev, const fsf_seq_desc* descs_host,
                  const int32_t* block_tables_dev, int32_t n_seqs, int32_t max_blocks, int32_t n_tokens,
                  void* out, void* workspace, void* hip_stream) {

  const Pass p = make_pass(cfg, descs_dev, block_tables_dev, n_seqs, max_blocks, n_tokens);
  hipStream_t stream = (hipStream_t)hip_stream;
  if (!fast_path_ok(cfg)) {
    const hipError_t e = fsf::launch_attn_generic(p, q, k_cache, v_cache, out, stream);
    return e == hipSuccess ? FSF_OK : FSF_ERR_HIP;
  }
  if (((uintptr_t)workspace & 255) != 0) return FSF_ERR_WORKSPACE;

  // ---- size the key cuts of the streaming sequences: enough items to fill the chip a few
  // times over, few enough that the partial results stay small next to the K/V traffic
  const int group = cfg->n_q_heads / cfg->n_kv_heads;
  int64_t dec_blocks = 0;  // cache blocks over all streaming units (every slice walks its sequence's blocks)
  for (int32_t s = 0; s < n_seqs; ++s) {
    const fsf_seq_desc& d = descs_host[s];
    if (!fsf::is_streaming(d.n_new, group, tn.stream_max_slices)) continue;
    int lo, hi, tmp;
    fsf::visible_range(d.n_cached, cfg->window, lo, tmp);
    fsf::visible_range(d.n_cached + d.n_new - 1, cfg->window, tmp, hi);
    dec_blocks += (int64_t)fsf::stream_slices(d.n_new, group) * (hi / cfg->block_size - lo / cfg->block_size + 1);
  }
  // Two rounds of the chip's 2048 wave slots: with the units launched longest first that is
  // balance enough, and every cut costs partial results whose writes are expensive.
  const int cus = tn.compute_units ? tn.compute_units : compute_units();
  const int min_item_blocks = tn.decode_min_item_blocks;
  const int64_t target_items = std::max<int64_t>(decode_target_items(cfg, tn), 1);  // 1: one item per slice, no cuts
  int64_t sb = (dec_blocks + target_items - 1) / target_items;
  if (sb < 1) sb = 1;

  const WsLayout w = ws_layout(cfg, tn, n_seqs, n_tokens);
  char* ws = (char*)workspace;
  fsf::FastPlan f;
  f.dec_item_start = (int32_t*)(ws + w.dec_item_start);
  f.pre_tile_start = (int32_t*)(ws + w.pre_tile_start);
  f.dec_prow_start = (int32_t*)(ws + w.dec_prow_start);
  f.dec_rec = (fsf::UnitRec*)(ws + w.dec_rec);
  f.pre_tile_seq = (int32_t*)(ws + w.pre_tile_seq);
  f.split_rows = (int32_t*)(ws + w.split_rows);
  f.part_ml = (float*)(ws + w.part_ml);
  f.part_acc = (float*)(ws + w.part_acc);
  f.split_blocks = (int32_t)std::min<int64_t>(sb, 1 << 30);
  f.min_item_blocks = min_item_blocks;
  f.stream_max_slices = tn.stream_max_slices;
  int64_t n_dec = 0, n_pre = 0, n_split_rows = 0, n_prows = 0, n_dec_cut = 0;  // n_dec_cut: items of sequences with cut keys
  auto count_work = [&] {
    n_dec = n_pre = n_split_rows = n_prows = n_dec_cut = 0;
    for (int32_t s = 0; s < n_seqs; ++s) {
      const fsf::SeqWork sw = fsf::seq_work(descs_host[s].n_new, descs_host[s].n_cached, cfg->window, cfg->block_size,
                                            group, f.stream_max_slices, f.split_blocks, f.min_item_blocks);
      n_dec += sw.dec_items;
      n_dec_cut += sw.cuts > 1 ? sw.dec_items : 0;
      n_pre += sw.pre_tiles;
      n_split_rows += sw.cuts > 1 ? descs_host[s].n_new : 0;
      n_prows += sw.prows;
    }
  };
  count_work();
  // A pass with so few streaming units that not even every compute unit gets a wave (one
  // long sequence alone, say) is bound by the latency of its longest unit: cut four times finer.
  if (n_dec * cfg->n_kv_heads < cus && !tn.min_item_blocks_given) {
    f.min_item_blocks = std::max(1, min_item_blocks / 4);
    count_work();
  }
  // With only a few rounds of the wave slots, a round that is barely begun still lasts as long as
  // a unit: 2.2 rounds of equal units take as long as 3.  Coarsen the cuts a little until the
  // units fill whole rounds.  Only where nearly all units come from cut sequences, so that they
  // are about equally long: in a pass of many uncut rows of all lengths and a few long cut ones,
  // longer cuts only lengthen the longest units (measured on the long-prompt stream: 1..4 % slower).
  if (tn.decode_hold == 1 && !tn.target_waves_given) {  // (a caller who names the number of units gets it)
    const int64_t slots = (int64_t)cus * 8;
    for (int it = 0; it < 16 && n_dec_cut * 5 >= n_dec * 4 && f.split_blocks < (1 << 28); ++it) {
      const int64_t units = n_dec * cfg->n_kv_heads;
      const int64_t full = units / slots, excess = units % slots;
      // fine as it is: whole rounds, a last round at least 80 % full, or so many rounds that one more hardly counts
      if (full < 1 || full >= 5 || excess == 0 || excess * 5 >= slots * 4) break;
      const int32_t before = f.split_blocks;
      f.split_blocks += std::max(1, f.split_blocks / 24);
      count_work();
      if (n_dec * cfg->n_kv_heads * 10 < full * slots * 9) {  // a step too far: a tenth of the last whole round left empty
        f.split_blocks = before;
        count_work();
        break;
      }
    }
  }
  // the partial results must fit their section: coarsen the cuts until they do (with cuts as
  // long as the longest sequence nothing is cut and nothing is needed)
  while (n_prows > (int64_t)w.prow_cap && f.split_blocks < (1 << 30)) {
    f.split_blocks *= 2;
    count_work();
  }
  if (n_prows > (int64_t)w.prow_cap || n_dec > (int64_t)w.items_cap) return FSF_ERR_WORKSPACE;  // cannot happen
  f.n_dec_items = (int32_t)n_dec;
  f.n_pre_tiles = (int32_t)n_pre;
  f.n_split_rows = (int32_t)n_split_rows;
  f.pre_part = (float*)(ws + w.pre_part);
  f.split = choose_prefill_split(cfg, tn, descs_host, n_seqs);
  f.decode_hold = tn.decode_hold;

  hipError_t e = fsf::launch_plan(p, f, stream);
  if (fused_launch(cfg)) {
    if (e == hipSuccess) e = fsf::launch_attn_fused(p, f, q, k_cache, v_cache, out, stream);
    if (e == hipSuccess) e = fsf::launch_prefill_merge(p, f, out, stream);
    if (e == hipSuccess) e = fsf::launch_attn_merge(p, f, out, stream);
    return e == hipSuccess ? FSF_OK : FSF_ERR_HIP;
  }
  // A pass with both kinds of work, and more streaming units than the chip has wave slots: the
  // prompt-chunk tiles run on the library's second stream, on the compute units the streaming
  // kernel leaves empty for them, forked after the planning and joined before the call returns
  // to the caller's stream.  Both kernels write disjoint rows of `out` and disjoint workspace.
  SideStream* side = nullptr;
  int reserve = 0;
  if (tn.overlap && tn.decode_hold == 1 && n_pre > 0 && n_dec * cfg->n_kv_heads > 8 * (int64_t)cus) {
    int64_t stream_bytes = 0;
    for (int32_t s = 0; s < n_seqs; ++s) {
      const fsf_seq_desc& d = descs_host[s];
      if (!fsf::is_streaming(d.n_new, group, tn.stream_max_slices)) continue;
      int lo, hi, tmp;
      fsf::visible_range(d.n_cached, cfg->window, lo, tmp);
      fsf::visible_range(d.n_cached + d.n_new - 1, cfg->window, tmp, hi);
      stream_bytes += (int64_t)fsf::stream_slices(d.n_new, group) * (hi - lo + 1) * cfg->n_kv_heads * fsf::kHeadDim * 4;
    }
    reserve = tn.overlap >= 8 ? std::min(tn.overlap, cus / 2 / 8 * 8)
                              : overlap_units(prefill_tile_steps_of(cfg, tn, descs_host, n_seqs), cfg->n_q_heads,
                                              stream_bytes, cus);
    side = reserve > 0 ? side_stream() : nullptr;
    if (!side) reserve = 0;
    // the tiles are cut for the units they will have
    if (side) {
      Tuning tside = tn;
      tside.compute_units = reserve;
      f.split = choose_prefill_split(cfg, tside, descs_host, n_seqs);
    }
  }
  if (side) {
    hipEvent_t fork, join;
    {
      std::lock_guard<std::mutex> lock(g_side_mutex);
      fork = side->fork[side->next % kSideEvents];
      join = side->join[side->next % kSideEvents];
      ++side->next;
    }
    if (e == hipSuccess) e = hipEventRecord(fork, stream);
    if (e == hipSuccess) e = hipStreamWaitEvent(side->stream, fork, 0);
    // `reserve` workgroups walk all tiles, the streaming kernel takes every other compute unit:
    // whichever kernel starts first, the chip is divided the same way
    if (e == hipSuccess) e = fsf::launch_attn_prefill(p, f, q, k_cache, v_cache, out, side->stream, reserve);
    if (e == hipSuccess) e = fsf::launch_prefill_merge(p, f, out, side->stream);
    // (the join is recorded even after an error, so that the caller's stream never waits on a
    // fork that nothing follows)
    const hipError_t ej = hipEventRecord(join, side->stream);
    if (e == hipSuccess) e = fsf::launch_attn_decode(p, f, q, k_cache, v_cache, out, stream, reserve);
    if (e == hipSuccess) e = fsf::launch_attn_merge(p, f, out, stream);
    const hipError_t ew = ej == hipSuccess ? hipStreamWaitEvent(stream, join, 0) : ej;
    if (e == hipSuccess) e = ew;
    return e == hipSuccess ? FSF_OK : FSF_ERR_HIP;
  }
  if (e == hipSuccess) e = fsf::launch_attn_prefill(p, f, q, k_cache, v_cache, out, stream);
  if (e == hipSuccess) e = fsf::launch_attn_decode(p, f, q, k_cache, v_cache, out, stream);
  if (e == hipSuccess) e = fsf::launch_prefill_merge(p, f, out, stream);
  if (e == hipSuccess) e = fsf::launch_attn_merge(p, f, out, stream);
  return e == hipSuccess ? FSF_OK : FSF_ERR_HIP;
}

}  // namespace

extern "C" int fsf_ragged_attention(const fsf_attn_cfg* cfg, const void* q, const void* k_cache,
                                    const void* v_cache, const fsf_seq_desc* descs_dev,
                                    const fsf_seq_desc* descs_host,
                                    const int32_t* block_tables_dev, int32_t n_seqs,
                                    int32_t max_blocks, int32_t n_tokens, void* out,
                                    void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (cfg_ok(cfg) && n_seqs == 0 && n_tokens == 0) return FSF_OK;
  const int st = attention_args_ok(cfg, q, k_cache, v_cache, descs_dev, descs_host, block_tables_dev, n_seqs,
                                   max_blocks, n_tokens, out);
  if (st != FSF_OK) return st;
  const size_t need = fsf_ragged_attention_workspace_bytes(cfg, n_seqs, n_tokens, max_blocks);
  if (!workspace || workspace_bytes < need) return FSF_ERR_WORKSPACE;
  return run_attention(cfg, resolve_tuning(cfg), q, k_cache, v_cache, descs_dev, descs_host, block_tables_dev,
                       n_seqs, max_blocks, n_tokens, out, workspace, hip_stream);
}

// ---------------------------------------------------------------------------------------------
// The same pass for callers that may not allocate: the work tables and partial results live in
// a fixed array in device memory that belongs to the library.  Every GPU the library runs on
// holds its own copy of the array at its own address, found once per device.
// ---------------------------------------------------------------------------------------------
namespace {

constexpr size_t kStaticScratchBytes = (size_t)FSF_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];  // device address of `scratch` on device i, once known

// Device address of this device's copy of `scratch` (the array's name is only a handle on the host).
void* static_scratch() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (p) return p;
  if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return nullptr;
  g_scratch_ptr[dev].store(p, std::memory_order_release);
  return p;
}

}  // namespace

extern "C" int fsf_ragged_attention_static(const fsf_attn_cfg* cfg, const void* q, const void* k_cache,
                                           const void* v_cache, const fsf_seq_desc* descs_dev,
                                           const fsf_seq_desc* descs_host, const int32_t* block_tables_dev,
                                           int32_t n_seqs, int32_t max_blocks, int32_t n_tokens, void* out,
                                           void* hip_stream) {
  if (cfg_ok(cfg) && n_seqs == 0 && n_tokens == 0) return FSF_OK;
  const int st = attention_args_ok(cfg, q, k_cache, v_cache, descs_dev, descs_host, block_tables_dev, n_seqs,
                                   max_blocks, n_tokens, out);
  if (st != FSF_OK) return st;
  Tuning tn = resolve_tuning(cfg);
  if (fast_path_ok(cfg)) {
    // partial results are what takes room: allow as many cut units as fit, down to none
    tn.max_decode_items_extra = std::min(tn.max_decode_items_extra, 1024);
    tn.max_prefill_split_units = std::min(tn.max_prefill_split_units, 64);
    while (ws_layout(cfg, tn, n_seqs, n_tokens).total > kStaticScratchBytes) {
      if (tn.max_decode_items_extra == 0 && tn.max_prefill_split_units == 0) return FSF_ERR_WORKSPACE;
      tn.max_decode_items_extra /= 2;
      tn.max_prefill_split_units /= 2;
    }
  }
  void* ws = static_scratch();
  if (!ws) return FSF_ERR_HIP;
  return run_attention(cfg, tn, q, k_cache, v_cache, descs_dev, descs_host, block_tables_dev, n_seqs,
                       max_blocks, n_tokens, out, ws, hip_stream);
}
