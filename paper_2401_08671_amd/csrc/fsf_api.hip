// C-ABI entry points: argument validation, path selection, launches.
//
// The entry points follow the paper's statement of the problem: a pass is a list of
// (tokens now, tokens cached) per sequence (Sec. 2) over a blocked cache (Sec. 2.1).
#include <stdlib.h>
#include <string.h>

#include <algorithm>

#include "fsf_internal.h"

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

// The matrix-core path takes 2-byte dtypes, head_dim 128, blocks of 64 * 2^k tokens (a 64-key
// step never straddles a block and finds its block with a shift), up to 16 query heads per
// KV head, and a cache block (all heads) below 4 GiB (its byte offsets are formed in 32-bit
// scalar multiplies).
bool fast_path_ok(const fsf_attn_cfg* c) {
  const int32_t steps_per_block = c->block_size / 64;
  return !(c->flags & FSF_FLAG_FORCE_GENERIC) && (c->dtype == FSF_BF16 || c->dtype == FSF_F16) &&
         c->head_dim == fsf::kHeadDim && c->block_size % 64 == 0 &&
         (steps_per_block & (steps_per_block - 1)) == 0 &&
         (uint64_t)c->n_kv_heads * c->block_size * fsf::kHeadDim * 2 < (1ull << 32) &&
         c->n_q_heads / c->n_kv_heads <= 16 && c->scale > 0.f;
}

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// Workspace sections of the matrix-core path, in order.
struct WsLayout {
  size_t dec_item_start, pre_tile_start, dec_item_seq, dec_order, pre_tile_seq, split_seqs, part_ml, part_acc, pre_part, total;
};

WsLayout ws_layout(const fsf_attn_cfg* c, int32_t n_seqs, int32_t n_tokens) {
  const size_t items_cap = (size_t)n_seqs + fsf::kMaxDecodeItemsExtra;
  const size_t tiles_cap = (size_t)n_seqs + (size_t)n_tokens / fsf::kPrefillTileM;
  WsLayout w;
  size_t off = 0;
  w.dec_item_start = off;
  off += align256(((size_t)n_seqs + 1) * sizeof(int32_t));
  w.pre_tile_start = off;
  off += align256(((size_t)n_seqs + 1) * sizeof(int32_t));
  w.dec_item_seq = off;
  off += align256(items_cap * sizeof(int32_t));
  w.dec_order = off;
  off += align256(items_cap * sizeof(int32_t));
  w.pre_tile_seq = off;
  off += align256(tiles_cap * sizeof(int32_t));
  w.split_seqs = off;
  off += align256(((size_t)n_seqs + 1) * sizeof(int32_t));
  w.part_ml = off;
  off += align256(items_cap * c->n_q_heads * 2 * sizeof(float));
  w.part_acc = off;
  off += align256(items_cap * c->n_q_heads * fsf::kHeadDim * sizeof(float));
  // partial results of split prompt-chunk tiles: at most kMaxPrefillSplitUnits (tile, head, part) workgroups
  const size_t split_units = std::min<size_t>(fsf::kMaxPrefillSplitUnits, tiles_cap * c->n_q_heads * 16);
  w.pre_part = off;
  off += align256(split_units * fsf::kPrefillTileM * fsf::kPrefillPartRowFloats * sizeof(float));
  w.total = off;
  return w;
}

int env_int(const char* name, int dflt) {
  const char* v = getenv(name);
  if (!v || !*v) return dflt;
  const int x = atoi(v);
  return x > 0 ? x : dflt;
}

int compute_units() {
  static int n = [] {
    int dev = 0, cu = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cu < 1)
      cu = 256;
    return cu;
  }();
  return n;
}

// Prompt-chunk workgroups (tile x head) are started heaviest first, one per compute unit at a
// time.  When the last round of them is less than half full (or there is less than one round),
// the tiles of that round are cut into parts along their keys so that the round fills the
// chip: f.pre_split_tiles tiles (the last to be started: tile indices 0 ..), f.pre_parts parts each.
void choose_prefill_split(const fsf_attn_cfg* c, const fsf_seq_desc* h, int32_t n_seqs, fsf::FastPlan& f) {
  f.pre_split_tiles = 0;
  f.pre_parts = 1;
  const int H = c->n_q_heads;
  const int cus = env_int("FSF_PREFILL_SPLIT_UNITS", compute_units());  // tests force splits with a large value
  if ((c->flags & FSF_FLAG_FUSED_LAUNCH) || f.n_pre_tiles == 0 || getenv("FSF_PREFILL_NO_SPLIT")) return;
  const int64_t groups = (int64_t)f.n_pre_tiles * H;
  const int64_t tail = groups % cus;  // workgroups of the last, partial round
  if (tail == 0 || 2 * tail > cus) return;
  // whole tiles only, and all of the partial round: an unsplit workgroup left in it would
  // last as long as the round did before
  int split_tiles = (int)((tail + H - 1) / H);
  if (split_tiles > f.n_pre_tiles) split_tiles = f.n_pre_tiles;
  int parts = std::max(2, (int)((cus + (int64_t)split_tiles * H / 2) / ((int64_t)split_tiles * H)));
  if ((int64_t)split_tiles * H * parts > fsf::kMaxPrefillSplitUnits)
    parts = (int)(fsf::kMaxPrefillSplitUnits / ((int64_t)split_tiles * H));
  // no part shorter than kPrefillMinPartSteps steps: look at the shortest of the tiles to split
  int tile = 0, min_steps = 1 << 30;
  for (int32_t s = 0; s < n_seqs && tile < split_tiles; ++s) {
    if (h[s].n_new == 1) continue;
    const int n_tiles = (h[s].n_new + fsf::kPrefillTileM - 1) / fsf::kPrefillTileM;
    for (int t = 0; t < n_tiles && tile < split_tiles; ++t, ++tile) {
      const int i0 = t * fsf::kPrefillTileM;
      const int i1 = std::min(i0 + fsf::kPrefillTileM, h[s].n_new);
      int lo, hi, tmp;
      fsf::visible_range(h[s].n_cached + i0, c->window, lo, tmp);
      fsf::visible_range(h[s].n_cached + i1 - 1, c->window, tmp, hi);
      min_steps = std::min(min_steps, (hi - (lo & ~63)) / 64 + 1);
    }
  }
  parts = std::min(std::min(parts, 16), min_steps / fsf::kPrefillMinPartSteps);
  if (parts < 2) return;
  f.pre_split_tiles = split_tiles;
  f.pre_parts = parts;
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

extern "C" int fsf_kv_append(const fsf_attn_cfg* cfg, const void* k_new, const void* v_new,
                             void* k_cache, void* v_cache, const fsf_seq_desc* descs_dev,
                             const int32_t* block_tables_dev, int32_t n_seqs, int32_t max_blocks,
                             int32_t n_tokens, void* hip_stream) {
  if (!cfg_ok(cfg) || n_seqs < 0 || n_tokens < 0 || max_blocks < 1) return FSF_ERR_INVALID_ARG;
  if (n_seqs == 0 || n_tokens == 0) return FSF_OK;
  if (!k_new || !v_new || !k_cache || !v_cache || !descs_dev || !block_tables_dev)
    return FSF_ERR_INVALID_ARG;
  if ((cfg->head_dim * elem_size(cfg)) % 4) return FSF_ERR_UNSUPPORTED;
  const Pass p = make_pass(cfg, descs_dev, block_tables_dev, n_seqs, max_blocks, n_tokens);
  const hipError_t e =
      fsf::launch_kv_append(p, k_new, v_new, k_cache, v_cache, (hipStream_t)hip_stream);
  return e == hipSuccess ? FSF_OK : FSF_ERR_HIP;
}

extern "C" size_t fsf_ragged_attention_workspace_bytes(const fsf_attn_cfg* cfg, int32_t n_seqs,
                                                       int32_t n_tokens, int32_t max_blocks) {
  if (!cfg_ok(cfg) || n_seqs < 0 || n_tokens < 0 || max_blocks < 1) return 0;
  if (!fast_path_ok(cfg)) return 256;
  return ws_layout(cfg, n_seqs, n_tokens).total;
}

extern "C" int fsf_ragged_attention(const fsf_attn_cfg* cfg, const void* q, const void* k_cache,
                                    const void* v_cache, const fsf_seq_desc* descs_dev,
                                    const fsf_seq_desc* descs_host,
                                    const int32_t* block_tables_dev, int32_t n_seqs,
                                    int32_t max_blocks, int32_t n_tokens, void* out,
                                    void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!cfg_ok(cfg) || n_seqs < 0 || n_tokens < 0 || max_blocks < 1) return FSF_ERR_INVALID_ARG;
  if (n_seqs == 0 && n_tokens == 0) return FSF_OK;
  if (!q || !k_cache || !v_cache || !descs_dev || !descs_host || !block_tables_dev || !out)
    return FSF_ERR_INVALID_ARG;
  if (!descs_ok(cfg, descs_host, n_seqs, max_blocks, n_tokens)) return FSF_ERR_INVALID_ARG;
  if (cfg->head_dim > 256) return FSF_ERR_UNSUPPORTED;
  const size_t need = fsf_ragged_attention_workspace_bytes(cfg, n_seqs, n_tokens, max_blocks);
  if (!workspace || workspace_bytes < need) return FSF_ERR_WORKSPACE;

  const Pass p = make_pass(cfg, descs_dev, block_tables_dev, n_seqs, max_blocks, n_tokens);
  hipStream_t stream = (hipStream_t)hip_stream;
  if (!fast_path_ok(cfg)) {
    const hipError_t e = fsf::launch_attn_generic(p, q, k_cache, v_cache, out, stream);
    return e == hipSuccess ? FSF_OK : FSF_ERR_HIP;
  }
  if (((uintptr_t)workspace & 255) != 0) return FSF_ERR_WORKSPACE;

  // ---- size the decode splits: enough items to fill the chip a few times over, few enough
  // that the partial results stay small next to the K/V traffic
  int64_t dec_blocks = 0;
  for (int32_t s = 0; s < n_seqs; ++s) {
    if (descs_host[s].n_new != 1) continue;
    int lo, hi;
    fsf::visible_range(descs_host[s].n_cached, cfg->window, lo, hi);
    dec_blocks += hi / cfg->block_size - lo / cfg->block_size + 1;
  }
  const int target_waves = env_int("FSF_DECODE_TARGET_WAVES", 16384);
  const int min_item_blocks = env_int("FSF_DECODE_MIN_ITEM_BLOCKS", 16);
  int64_t target_items = target_waves / cfg->n_kv_heads;
  if (target_items < 1) target_items = 1;
  if (target_items > fsf::kMaxDecodeItemsExtra) target_items = fsf::kMaxDecodeItemsExtra;
  int64_t sb = (dec_blocks + target_items - 1) / target_items;
  if (sb < 1) sb = 1;

  const WsLayout w = ws_layout(cfg, n_seqs, n_tokens);
  char* ws = (char*)workspace;
  fsf::FastPlan f;
  f.dec_item_start = (int32_t*)(ws + w.dec_item_start);
  f.pre_tile_start = (int32_t*)(ws + w.pre_tile_start);
  f.dec_item_seq = (int32_t*)(ws + w.dec_item_seq);
  f.dec_order = (int32_t*)(ws + w.dec_order);
  f.pre_tile_seq = (int32_t*)(ws + w.pre_tile_seq);
  f.split_seqs = (int32_t*)(ws + w.split_seqs);
  f.part_ml = (float*)(ws + w.part_ml);
  f.part_acc = (float*)(ws + w.part_acc);
  f.split_blocks = (int32_t)sb;
  f.min_item_blocks = min_item_blocks;
  int64_t n_dec = 0, n_pre = 0;
  int32_t n_split = 0;
  for (int32_t s = 0; s < n_seqs; ++s) {
    int d, t;
    fsf::seq_work(descs_host[s].n_new, descs_host[s].n_cached, cfg->window, cfg->block_size,
                  f.split_blocks, f.min_item_blocks, d, t);
    n_dec += d;
    n_pre += t;
    n_split += d > 1;
  }
  if (n_dec > (int64_t)n_seqs + fsf::kMaxDecodeItemsExtra) return FSF_ERR_WORKSPACE;  // cannot happen
  f.n_dec_items = (int32_t)n_dec;
  f.n_pre_tiles = (int32_t)n_pre;
  f.n_split_seqs = n_split;
  f.pre_part = (float*)(ws + w.pre_part);
  choose_prefill_split(cfg, descs_host, n_seqs, f);

  hipError_t e = fsf::launch_plan(p, f, stream);
  if (cfg->flags & FSF_FLAG_FUSED_LAUNCH) {
    if (e == hipSuccess) e = fsf::launch_attn_fused(p, f, q, k_cache, v_cache, out, stream);
  } else {
    if (e == hipSuccess) e = fsf::launch_attn_prefill(p, f, q, k_cache, v_cache, out, stream);
    if (e == hipSuccess) e = fsf::launch_attn_decode(p, f, q, k_cache, v_cache, out, stream);
  }
  if (e == hipSuccess) e = fsf::launch_prefill_merge(p, f, out, stream);
  if (e == hipSuccess) e = fsf::launch_attn_merge(p, f, out, stream);
  return e == hipSuccess ? FSF_OK : FSF_ERR_HIP;
}
