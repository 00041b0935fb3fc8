"""Matrix-core path (bf16/f16, head_dim 128, blocks of 16 * 2^k tokens) vs the fp64 oracle.

Element-by-element on shapes that span several tiles and ragged tails: generation rows
with and without KV splitting, prompt chunks with partial tiles and cached prefixes, GQA
groups 1..16, sliding windows cutting blocks, poisoned unwritten slots.
"""
import numpy as np
import pytest
import torch

from paper_2401_08671_amd import fsf
from paper_2401_08671_amd import workloads as wl
from tests.gpu_util import assert_cache_bit_exact, assert_outputs_close, run_hip
from tests.helpers import Step, plant_dominant_key

pytestmark = pytest.mark.gpu


def check_step(step, what="", flags=0, tuning=None):
    kc_o, vc_o, out_o = step.oracle()
    kc_h, vc_h, out_h = run_hip(step, flags=flags, tuning=tuning)
    assert_cache_bit_exact(kc_h, kc_o, what + " K")
    assert_cache_bit_exact(vc_h, vc_o, what + " V")
    return assert_outputs_close(out_h, out_o, step.spec.dtype, what)


def cut_rows(waves, min_blocks):
    """Tuning that forces fine cuts of the generation rows, so that the merge runs on short sequences too."""
    return fsf.Tuning(decode_target_waves=waves, decode_min_item_blocks=min_blocks)


def assume_units(units):
    """Tuning that pretends the chip has this many compute units, so that small batches get split tiles."""
    return fsf.Tuning(compute_units=units)


DECODE_LENS = [0, 1, 30, 31, 32, 33, 63, 64, 65, 127, 128, 200, 511, 512, 513, 1000, 2049]


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("heads", [(4, 4), (8, 2), (8, 1), (16, 1)])
@pytest.mark.parametrize("poison", ["nan", None])
def test_decode_rows(dtype, heads, poison):
    Hq, Hkv = heads
    spec = wl.BatchSpec("dec", Hq, Hkv, 128, 64, dtype, [(1, c) for c in DECODE_LENS], seed=9)
    check_step(Step(spec, poison=poison), f"decode {dtype} {heads} poison={poison}")


@pytest.mark.parametrize("split", [(1 << 20, 1), (1 << 20, 2), (64, 4)])
@pytest.mark.parametrize("window", [0, 100, 128, 1000])
def test_decode_rows_split_and_window(split, window):
    spec = wl.BatchSpec("decw", 8, 2, 128, 64, "bf16", [(1, c) for c in DECODE_LENS], window=window, seed=10)
    check_step(Step(spec, poison="nan"), f"decode split={split} window={window}", tuning=cut_rows(*split))


def test_decode_block_128():
    spec = wl.BatchSpec("dec128", 4, 2, 128, 128, "bf16", [(1, c) for c in (5, 127, 128, 300, 1025)],
                        seed=12)
    check_step(Step(spec, poison="inf"), "decode B=128")


PREFILL_SEQS = [(1, 5), (2, 0), (33, 0), (64, 64), (127, 1), (128, 0), (129, 63), (300, 200), (5, 1000)]


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("heads", [(2, 2), (8, 2)])
@pytest.mark.parametrize("window", [0, 70, 256])
def test_prefill_chunks(dtype, heads, window):
    Hq, Hkv = heads
    spec = wl.BatchSpec("pre", Hq, Hkv, 128, 64, dtype, PREFILL_SEQS, window=window, seed=13)
    check_step(Step(spec, poison="nan"), f"prefill {dtype} {heads} window={window}")


def test_prefill_long_chunk_over_long_prefix():
    spec = wl.BatchSpec("prelong", 2, 1, 128, 64, "bf16", [(700, 1500), (1, 2199)], seed=14)
    check_step(Step(spec, poison="nan"), "prefill 700 rows over 1500 cached")


@pytest.mark.parametrize("block", [128, 256])
def test_prefill_larger_blocks(block):
    """Several 64-key steps per cache block: the step -> block walk and the offset inside a block."""
    seqs = [(300, 900), (70, 0), (1, 300), (130, 129), (2, 511)]
    spec = wl.BatchSpec("preB", 4, 2, 128, block, "bf16", seqs, seed=21)
    check_step(Step(spec, poison="nan"), f"prefill block={block}")


@pytest.mark.parametrize("block", [16, 32])
@pytest.mark.parametrize("split", [(1 << 20, 1), (256, 4)])
@pytest.mark.parametrize("window", [0, 100, 1000])
def test_decode_rows_small_blocks(block, split, window):
    """Blocks of 16 and 32 tokens: a 32-key step spans two blocks (16) or is one block (32); unit
    boundaries then fall on multiples of 16 keys, inside a step."""
    spec = wl.BatchSpec("decsmall", 8, 2, 128, block, "bf16", [(1, c) for c in DECODE_LENS + [15, 16, 17, 47, 48]],
                        window=window, seed=25)
    check_step(Step(spec, poison="nan"), f"decode B={block} split={split} window={window}", tuning=cut_rows(*split))


@pytest.mark.parametrize("block", [16, 32])
@pytest.mark.parametrize("dtype,window", [("bf16", 0), ("f16", 70), ("bf16", 256)])
def test_prefill_small_blocks(block, dtype, window):
    """Blocks of 16 and 32 tokens: the four waves of a workgroup copy their 16 key rows of a step
    from different blocks; steps past the last token fall on blocks the sequence does not have."""
    seqs = PREFILL_SEQS + [(700, 1500), (130, 129), (17, 0), (16, 0), (1, 47), (49, 15)]
    spec = wl.BatchSpec("presmall", 4, 2, 128, block, dtype, seqs, window=window, seed=26)
    check_step(Step(spec, poison="nan"), f"prefill B={block} {dtype} window={window}")


@pytest.mark.parametrize("block", [16, 32])
def test_prefill_small_blocks_split_tiles(block):
    spec = wl.BatchSpec("presmallsplit", 2, 1, 128, block, "bf16", [(100, 3000), (300, 0), (1, 77)], seed=27)
    check_step(Step(spec, poison="nan"), f"prefill split B={block}", tuning=assume_units(64))


def test_prefill_block_192_takes_the_generic_kernel():
    """Blocks that are not 16 * 2^k tokens are served by the generic kernel, with the same results."""
    spec = wl.BatchSpec("pre192", 4, 2, 128, 192, "bf16", [(200, 300), (1, 500)], seed=22)
    check_step(Step(spec, poison="nan"), "prefill block=192")


def test_prefill_sharp_softmax_raises_the_reference_often():
    """A large logit scale makes row maxima jump by far more than 2^8 from step to step, so the
    running reference is raised (and the accumulators rescaled) inside the unmasked stretch too."""
    spec = wl.BatchSpec("presharp", 2, 1, 128, 64, "bf16", [(300, 2000), (140, 0)], seed=23, scale=0.7)
    check_step(Step(spec, poison="nan"), "prefill scale=0.7")


@pytest.mark.parametrize("window", [300, 1000])
def test_prefill_window_inside_long_prefix(window):
    """The visible range starts deep inside the cached prefix: leading steps are skipped, both
    ends of the range are masked, the stretch between them is not."""
    spec = wl.BatchSpec("prewin", 4, 1, 128, 64, "f16", [(260, 2000), (129, 700)], window=window, seed=24)
    check_step(Step(spec, poison="nan"), f"prefill window={window} over a long prefix")


@pytest.mark.parametrize("units,window,dtype", [(64, 0, "bf16"), (64, 700, "f16"), (40, 0, "bf16"), (1000, 0, "bf16")])
def test_prefill_tiles_split_along_keys(units, window, dtype):
    """Tiles of a partial last round are cut into parts along their keys (one workgroup each,
    unnormalised partial results, merge): forced here by a small unit count.  Parts that end
    before a row's first visible key, or start after its last, contribute nothing to that row."""
    seqs = [(700, 1500), (1, 900), (300, 2100), (1, 64)]
    spec = wl.BatchSpec("presplit", 2, 1, 128, 64, dtype, seqs, window=window, seed=31)
    check_step(Step(spec, poison="nan"), f"prefill split units={units} window={window} {dtype}", tuning=assume_units(units))


@pytest.mark.parametrize("heads,n_rows,block,dtype", [((16, 1), 5000, 64, "bf16"), ((8, 4), 1300, 64, "bf16"),
                                                      ((4, 4), 700, 64, "bf16"), ((8, 4), 1300, 16, "f16")])
@pytest.mark.parametrize("hold", [0, 2, -1])
def test_more_generation_row_units_than_wave_slots(heads, n_rows, block, dtype, hold):
    """With more units than resident waves the generation-row kernel runs as one round of waves
    that walk several units each and hold their results in LDS until the end: 16 heads per KV head
    leave room for two held units (stored whenever both slots are full), 2 heads for all of them;
    the third shape stays below the wave slots and takes the one-unit-per-workgroup form.  hold 0:
    eight-wave workgroups, one per compute unit (consecutive launch slots where a workgroup covers
    whole sequences' KV heads, strided otherwise); 2: single-wave workgroups; -1: nothing held."""
    Hq, Hkv = heads
    rng = np.random.default_rng(36)
    seqs = [(1, int(c)) for c in rng.integers(0, 200, size=n_rows)]
    seqs[7] = (1, 5000)                       # one long row: cut into units with partial results
    spec = wl.BatchSpec("manyunits", Hq, Hkv, 128, block, dtype, seqs, seed=36)
    check_step(Step(spec, poison="nan"), f"{n_rows} rows, heads {heads}, block {block}, {dtype}, hold {hold}",
               tuning=fsf.Tuning(decode_hold=hold))


@pytest.mark.parametrize("units", [1, 32])
@pytest.mark.parametrize("heads", [(8, 2), (40, 40), (6, 3)])
def test_prompt_chunks_beside_the_streaming_kernel(heads, units):
    """overlap = 1 (compute units from the cost model) or 32 (exactly that many): the prompt-chunk
    tiles run on the library's second stream, walked by a few persistent workgroups, while the
    streaming kernel leaves those compute units empty; forked and joined inside the call.  Two
    passes back to back without a wait in between, then the same pass again: equal bits, and the
    oracle's result."""
    Hq, Hkv = heads
    rng = np.random.default_rng(88)
    seqs = [(1, int(c)) for c in rng.integers(0, 400, size=1500)] + [(300, 100), (40, 3), (700, 0), (1, 3000)]
    spec = wl.BatchSpec("overlap", Hq, Hkv, 128, 64, "bf16", seqs, seed=88)
    st = Step(spec, poison="nan")
    tn = fsf.Tuning(overlap=units)
    _, _, ref = st.oracle()
    _, _, a = run_hip(st, tuning=tn, return_cache=False)
    _, _, b = run_hip(st, tuning=tn, return_cache=False, repeat_attention=3)
    assert_outputs_close(a, ref, "bf16", f"overlap {units} heads {heads}")
    assert np.array_equal(a, b)
    if units == 1:   # (a given number of units cuts the tiles for that many: another summation order)
        _, _, c = run_hip(st, tuning=fsf.Tuning(overlap=-1), return_cache=False)
        assert np.array_equal(a, c), "the partition of the work is the same with and without the second stream"


@pytest.mark.parametrize("heads", [(3, 1), (10, 2), (12, 2), (36, 3), (15, 1)])
@pytest.mark.parametrize("block", [16, 64])
def test_head_groups_that_are_no_power_of_two(heads, block):
    """3, 5, 6, 12 and 15 query heads per KV head: a slice of the streaming kernel then holds
    16 // group rows and leaves columns unused; generation rows, short chunks on the streaming
    kernel (cut and whole) and tiled chunks in one pass."""
    Hq, Hkv = heads
    rng = np.random.default_rng(Hq * 100 + block)
    seqs = [(1, int(c)) for c in rng.integers(0, 2500, size=40)] + [(2, 700), (5, 0), (11, 3000), (31, 64), (300, 500)]
    seqs = [seqs[i] for i in rng.permutation(len(seqs))]
    spec = wl.BatchSpec("oddgroup", Hq, Hkv, 128, block, "bf16", seqs, seed=500 + Hq)
    st = Step(spec, poison="nan")
    check_step(st, f"heads {heads} block {block}", tuning=fsf.Tuning(stream_chunk_slices=16))
    check_step(st, f"heads {heads} block {block}, rows cut", tuning=cut_rows(1 << 20, 256 // block))


def test_fifty_thousand_sequences():
    """A pass of 50 000 short generation rows and two chunks: the planning kernel's prefix sums and
    counting sort over many sequences per thread, 100 000 units for 2048 wave slots."""
    rng = np.random.default_rng(5)
    seqs = [(1, int(c)) for c in rng.integers(0, 16, size=50000)] + [(40, 3), (300, 0)]
    spec = wl.BatchSpec("many", 2, 2, 128, 16, "bf16", seqs, seed=9)
    check_step(Step(spec, poison="nan"), "50000 sequences")


@pytest.mark.parametrize("window", [0, 5000])
def test_very_long_contexts(window):
    """A generation row over 200 000 cached tokens (cut into many units and merged) and a 300-row
    chunk over 150 000: long block tables, large offsets, thousands of steps per tile."""
    spec = wl.BatchSpec("long", 2, 1, 128, 64, "bf16", [(1, 200_000), (300, 150_000), (1, 70_001)], window=window, seed=34)
    check_step(Step(spec), f"long contexts window={window}")


@pytest.mark.parametrize("given", [False, True])
def test_few_long_rows_cut_by_the_default_rules(given):
    """100 rows over 8000..16000 cached tokens with 8 KV heads: every row is cut, the units come to
    a little over two rounds of the wave slots, and the default rules then cut a little coarser so
    that the units fill two rounds (a named number of units is taken as given).  Whatever the
    cuts, the oracle's result."""
    rng = np.random.default_rng(12)
    seqs = [(1, int(c)) for c in rng.integers(8000, 16000, size=100)]
    spec = wl.BatchSpec("fewlong", 8, 8, 128, 64, "bf16", seqs, seed=77)
    check_step(Step(spec), f"few long rows, units given: {given}",
               tuning=fsf.Tuning(decode_target_waves=4096) if given else None)


@pytest.mark.parametrize("mult", [1.0, 1.0 / np.sqrt(128.0)])
@pytest.mark.parametrize("block", [16, 64])
def test_every_unit_of_a_cut_generation_row_counts(mult, block):
    """Rows over 12 000 cached tokens, cut into units of 256 keys.  In sequence u one key inside
    unit 3u (and the first and the last key in two more sequences) is given a dominant logit, so
    that row's output is that key's V row: a unit that is lost, merged with the wrong weight or
    counted twice moves it by O(1).  Also with values scaled like benchmark shape 2, where
    ordinary outputs lie below the absolute tolerance."""
    c, per_unit = 12_000, 256
    n_units = -(-(c + 1) // per_unit)
    plants = [min(3 * u * per_unit + 17 * u + 5, c) for u in range(0, (n_units + 2) // 3)] + [0, c, per_unit - 1, per_unit]
    spec = wl.BatchSpec("plantdec", 2, 1, 128, block, "bf16", [(1, c)] * len(plants), value_mult=mult, seed=41)
    st = Step(spec)
    want_v = [plant_dominant_key(st, s, 0, 0, pos) for s, pos in enumerate(plants)]
    tn = cut_rows(1 << 20, per_unit // block)
    _, _, out_o = st.oracle()
    _, _, out_h = run_hip(st, tuning=tn, return_cache=False)
    assert_outputs_close(out_h, out_o, "bf16", f"planted keys mult={mult:.3f} B={block}")
    for s, v in enumerate(want_v):
        assert np.abs(out_o[s, 0] - v).max() <= 1e-9 * max(1.0, np.abs(v).max()), "the plant did not take"
        assert np.abs(out_h[s, 0] - v).max() <= 2.0 ** -8 * np.abs(v).max() + 1e-30, f"sequence {s}, key {plants[s]}"


@pytest.mark.parametrize("units,window", [(64, 0), (1000, 0), (64, 2500)])
def test_every_part_of_a_split_tile_counts(units, window):
    """A 300-row chunk over 3000 cached tokens whose tiles are cut into parts along their keys.
    Sixteen of its rows get one dominant key each, spread over the whole visible range, so every
    part holds the dominant key of some row."""
    n, c = 300, 3000
    spec = wl.BatchSpec("plantpre", 2, 1, 128, 64, "bf16", [(n, c), (1, 77)], window=window, seed=42)
    st = Step(spec)
    rows = [n - 1 - 18 * k for k in range(16)]
    plants = []
    for k, r in enumerate(rows):
        lo = max(0, c + r - window + 1) if window else 0
        pos = lo + (c + r - lo) * k // 15                  # from the row's first visible key to its own
        plants.append((r, pos, plant_dominant_key(st, 0, r, 0, pos)))
    _, _, out_o = st.oracle()
    _, _, out_h = run_hip(st, tuning=assume_units(units), return_cache=False)
    assert_outputs_close(out_h, out_o, "bf16", f"planted keys in a split tile units={units} window={window}")
    for r, pos, v in plants:
        assert np.abs(out_o[r, 0] - v).max() <= 1e-9 * np.abs(v).max(), "the plant did not take"
        assert np.abs(out_h[r, 0] - v).max() <= 2.0 ** -8 * np.abs(v).max(), f"row {r}, key {pos}"


SHORT_PREFIXES = [0, 5, 63, 64, 700, 31, 1, 129]


@pytest.mark.parametrize("group", [1, 4, 8, 16])
@pytest.mark.parametrize("window", [0, 100])
@pytest.mark.parametrize("block", [16, 64])
def test_short_chunks_on_the_streaming_kernel(group, window, block):
    """Chunks of 2..17 rows (what filling the token budget exactly leaves at the end of a pass,
    and the remainders of prompts) run on the streaming kernel with (row, head) pairs in the 16
    columns of a unit, every column with its own causal and window bound: one slice for 16 / group
    rows, several slices beyond.  Interleaved with an ordinary chunk and generation rows."""
    seqs = []
    for n in range(2, 18):
        seqs.append((n, SHORT_PREFIXES[n % len(SHORT_PREFIXES)]))
        if n % 5 == 0:
            seqs.append((1, 40 * n))
    seqs.insert(7, (300, 90))
    spec = wl.BatchSpec("short", 2 * group, 2, 128, block, "bf16" if group != 4 else "f16", seqs, window=window, seed=60 + group)
    tn = fsf.Tuning(stream_chunk_slices=16)
    check_step(Step(spec, poison="nan"), f"short chunks g={group} W={window} B={block}", tuning=tn)


@pytest.mark.parametrize("slices", [-1, 0, 1, 3])
def test_short_chunks_either_kernel_gives_the_oracle_result(slices):
    """The same pass with short chunks on the tiled kernel (-1), by the default rule (0: up to two
    slices stream) and with other limits."""
    seqs = [(2, 1000), (1, 77), (8, 3), (9, 640), (16, 0), (17, 200), (31, 64), (40, 500), (1, 0)]
    spec = wl.BatchSpec("either", 8, 2, 128, 64, "bf16", seqs, seed=66)
    check_step(Step(spec, poison="nan"), f"stream_chunk_slices={slices}", tuning=fsf.Tuning(stream_chunk_slices=slices))


@pytest.mark.parametrize("group,window,block", [(1, 0, 64), (4, 0, 64), (4, 3000, 16), (16, 0, 64)])
def test_short_chunks_with_cut_keys_every_cut_counts(group, window, block):
    """Short chunks over long prefixes whose keys are cut into units of 128 keys with partial results
    for every (cut, row): rows of a slice see different numbers of cuts (a cut past a row's own
    position holds nothing for it), early slices see none of the last cuts.  One key in every
    third cut is made dominant for one row of the chunk in turn."""
    n, c = 14, 5000
    spec = wl.BatchSpec("shortcut", 2 * group, 2, 128, block, "bf16", [(n, c), (1, 300), (5, 4990), (n, 70)],
                        window=window, seed=70 + group)
    st = Step(spec, poison="nan")
    plants = []
    for k in range(12):
        r = (5 * k) % n
        lo = max(0, c + r - window + 1) if window else 0
        pos = lo + (c + r - lo) * k // 11
        plants.append((r, pos, plant_dominant_key(st, 0, r, 0, pos)))
    tn = fsf.Tuning(stream_chunk_slices=16, decode_target_waves=1 << 20, decode_min_item_blocks=128 // block)
    _, _, out_o = st.oracle()
    _, _, out_h = run_hip(st, tuning=tn, return_cache=False)
    assert_outputs_close(out_h, out_o, "bf16", f"short chunk with cut keys g={group} W={window} B={block}")
    for r, pos, v in plants[-3:]:          # the last plants of a row are the ones no later plant overrides
        assert np.abs(out_o[r, 0] - v).max() <= 1e-6 * np.abs(v).max(), "the plant did not take"
        assert np.abs(out_h[r, 0] - v).max() <= 2.0 ** -8 * np.abs(v).max(), f"row {r}, key {pos}"


def test_thousands_of_two_row_chunks():
    """Many short chunks and generation rows: more streaming units than wave slots, so waves walk
    several units each; one-row units hold their results back, chunk units store at once."""
    rng = np.random.default_rng(77)
    seqs = [((2 if i % 3 else 1), int(c)) for i, c in enumerate(rng.integers(0, 150, size=2400))]
    seqs[11] = (3, 4000)
    spec = wl.BatchSpec("manyshort", 4, 4, 128, 64, "bf16", seqs, seed=77)
    check_step(Step(spec, poison="nan"), "2400 short sequences")


@pytest.mark.parametrize("flags", [0, fsf.FSF_FLAG_FUSED_LAUNCH])
def test_mixed_batch_order_independent(flags):
    """Chunks and generations interleaved in any order (the kernels may not assume chunks come first);
    also through the single fused launch."""
    seqs = [(1, 77), (150, 10), (1, 640), (3, 0), (1, 0), (260, 300), (1, 129), (700, 40)]
    spec = wl.BatchSpec("mix", 8, 8, 128, 64, "bf16", seqs, seed=15)
    check_step(Step(spec, poison="nan"), f"mixed order flags={flags}", flags=flags)


@pytest.mark.parametrize("k,nd", [(2, 24), (4, 40)])
def test_benchmark_shapes_reduced_fused_launch(k, nd):
    spec = wl.config(k, n_decodes=nd)
    if k == 2:
        spec.seqs = [(448, 0)] + spec.seqs[1:]
    check_step(Step(spec), f"cfg{k} reduced, fused launch", flags=fsf.FSF_FLAG_FUSED_LAUNCH)


def test_fast_path_matches_generic_kernel_within_tolerance():
    """Two independent device paths agree (both are also checked against the oracle above)."""
    spec = wl.BatchSpec("xchk", 8, 2, 128, 64, "bf16", [(100, 30), (1, 500), (1, 64)], seed=16)
    st = Step(spec)
    _, _, fast = run_hip(st)
    _, _, gen = run_hip(st, flags=fsf.FSF_FLAG_FORCE_GENERIC)
    assert np.abs(fast - gen).max() <= 2e-2


def test_results_are_deterministic():
    spec = wl.BatchSpec("det", 8, 2, 128, 64, "bf16", [(200, 100)] + [(1, c) for c in (900, 64, 3000)], seed=17)
    st = Step(spec)
    _, _, a = run_hip(st)
    _, _, b = run_hip(st)
    assert np.array_equal(a, b)


@pytest.mark.parametrize("k,nd", [(2, 24), (3, 48), (4, 40)])
def test_benchmark_shapes_reduced(k, nd):
    """Benchmark shapes 2-4 with fewer generation rows: full element-wise parity."""
    spec = wl.config(k, n_decodes=nd)
    if k == 3:      # keep the oracle's dense score matrices small: shorter prefixes, same window logic
        spec.seqs = [(256, 2048), (256, 6144)] + spec.seqs[2:]
    if k == 2:
        spec.seqs = [(448, 0)] + spec.seqs[1:]
    check_step(Step(spec), f"cfg{k} reduced")


@pytest.mark.parametrize("seed", range(10))
def test_random_ragged_batches(seed):
    """Seeded random passes: chunks of any length over any prefix next to generation rows, random
    head grouping, window, block size and unit count (which moves the split rules around)."""
    rng = np.random.default_rng(7000 + seed)
    Hkv = int(rng.choice([1, 2, 4]))
    Hq = Hkv * int(rng.choice([1, 2, 4, 8]))
    block = int(rng.choice([64, 64, 128]))
    window = int(rng.choice([0, 0, 0, 90, 1000]))
    dtype = "bf16" if seed % 3 else "f16"
    seqs = []
    for _ in range(int(rng.integers(1, 5))):          # prompt chunks
        n = int(rng.choice([2, 17, 64, 200, 256, 257, 600, 1100]))
        c = int(rng.choice([0, 0, 5, 63, 64, 700, 3000]))
        seqs.append((n, c))
    for _ in range(int(rng.integers(0, 6))):          # generation rows
        seqs.append((1, int(rng.choice([0, 1, 63, 64, 500, 2000]))))
    order = rng.permutation(len(seqs))
    seqs = [seqs[i] for i in order]
    # keep the oracle's dense score matrices small
    assert sum((n + c) * n for n, c in seqs) < 30_000_000
    tn = assume_units(int(rng.choice([4, 16, 64, 256])))
    spec = wl.BatchSpec(f"rand{seed}", Hq, Hkv, 128, block, dtype, seqs, window=window, seed=8000 + seed)
    check_step(Step(spec, poison="nan"), f"random batch {seed}: Hq={Hq} Hkv={Hkv} B={block} W={window} {dtype} {seqs}", tuning=tn)


@pytest.mark.parametrize("overlap", [0, 1])
def test_a_pass_can_be_captured_in_a_graph_and_replayed(overlap):
    """Append + attention of a mixed pass recorded into a HIP graph (the library allocates nothing,
    clears nothing with memset and waits for nothing): every replay, with eager work and
    synchronisation in between, gives the bits of the eager run, which is checked against the oracle."""
    from paper_2401_08671_amd.harness import DeviceStep
    seqs = [(300, 100), (1, 2000), (1, 63), (700, 0), (1, 5000)]
    if overlap:          # enough generation rows for the one-round streaming grid, so that the fork to the
        seqs += [(1, 40 + (7 * i) % 300) for i in range(1200)]      # second stream is part of the recorded graph
    spec = wl.BatchSpec("graph", 8, 2, 128, 64, "bf16", seqs, seed=35)
    ds = DeviceStep(spec, tuning=fsf.Tuning(overlap=overlap))
    ds.step()
    torch.cuda.synchronize()
    eager = ds.out.clone()
    k_after, v_after = ds.k_cache.clone(), ds.v_cache.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):          # warm-up on the capture stream
        ds.step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        ds.step()
    torch.cuda.synchronize()
    for r in range(4):
        ds.out.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(ds.out, eager), f"replay {r}"
        assert torch.equal(ds.k_cache, k_after) and torch.equal(ds.v_cache, v_after)
        assert float(ds.q.float().abs().sum()) > 0      # eager work between the replays
    # and the eager result itself is right
    kc = wl.to_numpy_storage(ds.k_cache)
    vc = wl.to_numpy_storage(ds.v_cache)
    from oracle import attention as oa
    ref = oa.ragged_attention(wl.to_numpy_storage(ds.q), kc, vc, ds.descs, ds.block_tables, block_size=64,
                              scale=spec.scale, window=0, dtype="bf16")
    assert_outputs_close(eager.to(torch.float64).cpu().numpy(), ref, "bf16", "graph pass")


@pytest.mark.parametrize("seed", range(100, 112))
def test_random_passes_over_block_sizes_groups_and_unit_counts(seed):
    """Seeded random passes over the whole matrix-core envelope: 1 to 16 query heads per KV head,
    blocks of 16 to 128 tokens, windows, no to thousands of generation rows (one unit per workgroup,
    or one round of waves holding their results), forced fine or no cuts of the rows."""
    rng = np.random.default_rng(seed)
    Hkv = int(rng.choice([1, 2, 4]))
    Hq = Hkv * int(rng.choice([1, 2, 4, 8, 16]))
    block = int(rng.choice([16, 32, 64, 128]))
    window = int(rng.choice([0, 0, 90, 1000]))
    dtype = "bf16" if seed % 3 else "f16"
    seqs = []
    for _ in range(int(rng.integers(0, 4))):
        seqs.append((int(rng.choice([2, 17, 64, 200, 256, 257, 600])), int(rng.choice([0, 5, 63, 64, 700, 3000]))))
    n_dec = int(rng.choice([0, 3, 40, 700, 2500]))
    seqs += [(1, int(c)) for c in rng.integers(0, int(rng.choice([40, 300, 3000])), size=n_dec)]
    if not seqs:
        seqs = [(1, 5)]
    order = rng.permutation(len(seqs))
    seqs = [seqs[i] for i in order]
    tn = assume_units(int(rng.choice([4, 16, 64, 256])))
    if rng.random() < 0.3:
        tn.decode_target_waves, tn.decode_min_item_blocks = int(rng.choice([64, 100000])), 16
    spec = wl.BatchSpec(f"wide{seed}", Hq, Hkv, 128, block, dtype, seqs, window=window, seed=9000 + seed)
    check_step(Step(spec, poison="nan"), f"seed {seed}: Hq={Hq} Hkv={Hkv} B={block} W={window} {dtype} n_seqs={len(seqs)}", tuning=tn)
