"""CPU-side checks of the boundary: the library loads, exports every symbol the header
declares, answers the size queries, and rejects bad descriptions without touching a GPU."""
import ctypes
import os
import re

import paper_2508_15212_amd as spark
from paper_2508_15212_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    names = set()
    for header in ("spark.h", "spark_bench.h"):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(spark_[a-z_0-9]+)\s*\(", text))
    return sorted(names)


def test_the_method_header_holds_no_measurement_aid():
    text = open(os.path.join(ROOT, "include", "spark.h")).read()
    assert "spark_probe_read" not in text


def test_library_exports_every_declared_symbol():
    lib = spark.load()
    names = _declared()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def _desc(**kw):
    d = spark.SparkDesc(batch=8, n_q_heads=32, n_kv_heads=8, head_dim=128, keep=26, window=32,
                        total_tokens=8 * 32768, k_token_stride=128, k_head_stride=128 * 8 * 32768,
                        v_token_stride=128, v_head_stride=128 * 8 * 32768)
    for k, v in kw.items():
        setattr(d, k, v)
    return d


def test_size_queries_follow_the_layout():
    d = _desc()
    rows = 8 * 32768 * 8
    # 72-byte rows at T = 26 (13 value words + 4 mask words + mu), plus header and a / 1/a
    assert spark.packed_bytes(d) == 256 + 2 * 8 * 8 * 128 * 4 + rows * 72
    assert spark.packed_bytes(_desc(keep=64)) == 256 + 2 * 8 * 8 * 128 * 4 + rows * 152
    assert spark.packed_bytes(_desc(pack_dtype=spark.PACK_INT8)) == 256 + 2 * 8 * 8 * 128 * 4 + rows * 56
    ns = spark.decode_splits(d)
    assert ns >= 1
    assert ns == 8                          # 4096 tiles x 8 heads / 512 blocks = chunks of 64 tiles; 512 / 64
    # slots: one per (chunk, q head) for at most (4096 + 2 * 8) // 64 + 8 + 1 = 73 chunks, plus one spare per
    # (batch, q head) for appended rows; 130 floats per slot; then the 8 * 8 arrival counters
    # (the counters come first, padded to 256 bytes, so their place depends on batch and KV heads only)
    assert spark.decode_workspace_bytes(d) == (73 * 32 + 8 * 32 * 1) * 130 * 4 + 256
    assert spark.decode_workspace_bytes(_desc(batch=64, total_tokens=64 * 2048)) % 256 == 0
    assert spark.decode_splits(_desc(n_splits=7)) == 7
    # partial last tile is padded to 64 tokens
    assert spark.packed_bytes(_desc(batch=1, total_tokens=65)) == 256 + 2 * 8 * 128 * 4 + 2 * 64 * 8 * 72


def test_balanced_cut_sizes_its_partial_slots_on_the_host():
    """n_splits = -1 asks for the balanced cut: 4 * (512 / KV heads) wavefronts per KV head, chunk ids
    wavefronts + 2 * batch.  Batches of 32 to 256 sequences with 256 or more (batch, KV head) pairs and two
    tiles or more per wavefront get it unasked; more than 256 sequences, or 16 query heads per KV head, never do."""
    slot = 130 * 4
    small = _desc(batch=4, total_tokens=4 * 1000)
    forced = _desc(batch=4, total_tokens=4 * 1000, n_splits=-1)
    assert spark.decode_workspace_bytes(forced) == ((256 + 2 * 4) * 32 + 4 * 32) * slot + 256
    assert spark.decode_workspace_bytes(forced) > spark.decode_workspace_bytes(small)
    assert spark.decode_splits(forced) == 0 and spark.decode_splits(small) >= 1     # (0: the balanced cut)
    ragged = _desc(batch=64, total_tokens=64 * 1300)
    assert spark.decode_workspace_bytes(ragged) == ((256 + 2 * 64) * 32 + 64 * 32) * slot + 64 * 8 * 4
    assert spark.decode_workspace_bytes(_desc(batch=64, total_tokens=64 * 1300, n_splits=-1)) == \
        spark.decode_workspace_bytes(ragged)
    # a fixed split count switches it off; so do 16 query heads per KV head and more than 256 sequences
    assert spark.decode_workspace_bytes(_desc(batch=64, total_tokens=64 * 1300, n_splits=1)) == \
        (64 * 32 + 64 * 32) * slot + 64 * 8 * 4
    wide = dict(n_q_heads=128, n_kv_heads=8, batch=4, total_tokens=4 * 1000)
    assert spark.decode_workspace_bytes(_desc(n_splits=-1, **wide)) == spark.decode_workspace_bytes(_desc(**wide))
    many = dict(batch=300, total_tokens=300 * 100)
    assert spark.decode_workspace_bytes(_desc(n_splits=-1, **many)) == spark.decode_workspace_bytes(_desc(**many))
    # the caller's hint: a longest sequence within 9/8 of the average keeps one block per sequence
    # (chunks of 2 * ceil(1300 tiles * 8 heads / 512) = 42 tiles: at most (1300 + 128) // 42 + 64 + 1 = 99 of them)
    by_length = (99 * 32 + 64 * 32) * slot + 64 * 8 * 4
    assert spark.decode_workspace_bytes(_desc(batch=64, total_tokens=64 * 1300, max_seqlen=1400)) == by_length
    assert spark.decode_workspace_bytes(_desc(batch=64, total_tokens=64 * 1300, max_seqlen=1463)) > by_length
    assert spark.decode_workspace_bytes(_desc(batch=64, total_tokens=64 * 1300, max_seqlen=1400, n_splits=-1)) > by_length
    # ... and a batch with less than two tiles per wavefront (here 400 tiles for 256 wavefronts) is left alone
    assert spark.decode_splits(_desc(batch=64, total_tokens=64 * 400)) >= 1
    assert spark.decode_splits(_desc(batch=64, total_tokens=64 * 400, n_splits=-1)) == 0
    assert spark.decode_workspace_bytes(_desc(max_seqlen=-1)) == 0
    assert spark.decode_workspace_bytes(_desc(n_splits=-2)) == 0
    assert spark.decode_workspace_bytes(_desc(n_splits=4097)) == 0


def test_bad_descriptions_are_rejected_on_the_host():
    lib = spark.load()
    assert spark.packed_bytes(_desc(head_dim=64)) == 0
    assert spark.packed_bytes(_desc(keep=0)) == 0
    assert spark.packed_bytes(_desc(keep=129)) == 0
    assert spark.packed_bytes(_desc(n_q_heads=24, n_kv_heads=8)) == 0      # group of 3
    assert spark.packed_bytes(_desc(n_q_heads=30)) == 0
    # NULL pointers are caught before any launch (status 1 = invalid argument)
    d = _desc()
    assert lib.spark_prune(ctypes.byref(d), None, None, None, None, None, 0, None) == 1
    assert lib.spark_decode_attn(ctypes.byref(d), None, None, None, None, None, None, 0, None) == 1
    assert lib.spark_unpack(ctypes.byref(d), None, None, None, None, None, None, None) == 1
    assert lib.spark_prune(ctypes.byref(_desc(head_dim=64)), None, None, None, None, None, 0, None) == 2
    assert lib.spark_status_string(3) == b"workspace too small"


def test_alignment_strides_and_workspace_are_checked_before_any_launch():
    """Fake (never dereferenced) device addresses: every one of these calls must fail on the host."""
    lib = spark.load()
    d = _desc()
    A = 0x7F0000000000            # 256-byte aligned fake address
    ok_ws = spark.decode_workspace_bytes(d)
    # misaligned packed buffer / V pointer / workspace
    assert lib.spark_prune(ctypes.byref(d), A, A, A, A + 64, None, 0, None) == 1
    assert lib.spark_decode_attn(ctypes.byref(d), A, A + 8, A, A, A, A, ok_ws, None) == 1
    assert lib.spark_decode_attn(ctypes.byref(d), A, A, A + 2, A, A, A, ok_ws, None) == 1
    assert lib.spark_decode_attn(ctypes.byref(d), A, A, A, A, A, A + 4, ok_ws, None) == 1
    # workspace one byte short
    assert lib.spark_decode_attn(ctypes.byref(d), A, A, A, A, A, A, ok_ws - 1, None) == 3
    assert lib.spark_decode_workspace_init(ctypes.byref(d), A, ok_ws - 1, None) == 3
    # strides that would break 16-byte row alignment, or rows that overlap
    assert lib.spark_prune(ctypes.byref(_desc(k_token_stride=130)), A, A, A, A, None, 0, None) == 1
    assert lib.spark_prune(ctypes.byref(_desc(k_token_stride=64)), A, A, A, A, None, 0, None) == 1
    assert lib.spark_decode_attn(ctypes.byref(_desc(v_head_stride=100)), A, A, A, A, A, A, ok_ws, None) == 1
    assert lib.spark_prune(ctypes.byref(_desc(window=0)), A, A, A, A, None, 0, None) == 1
    assert lib.spark_probe_read(None, 1024, A, 4, None) == 1
    assert lib.spark_probe_read(A, 8, A, 4, None) == 1
    # K and V base pointers must be 16-byte aligned (the kernels issue 4- and 16-byte row loads)
    assert lib.spark_prune(ctypes.byref(d), A + 2, A, A, A, None, 0, None) == 1
    assert lib.spark_prune(ctypes.byref(d), A + 8, A, A, A, None, 0, None) == 1
    assert lib.spark_prune_values(ctypes.byref(_desc(keep_v=64)), A + 4, A, None) == 1
    # the cache checker rejects bad arguments before it copies anything
    assert lib.spark_check_packed(ctypes.byref(d), None, 0, None) == 1
    assert lib.spark_check_packed(ctypes.byref(d), A + 64, 0, None) == 1
    assert lib.spark_check_packed(ctypes.byref(d), A, 1, None) == 1          # keep_v = 0: there is no value cache
    assert lib.spark_check_packed(ctypes.byref(_desc(head_dim=64)), A, 0, None) == 2
    assert lib.spark_status_string(5) == b"packed cache does not match the description"


def test_value_cache_and_tail_entry_points_check_their_arguments_on_the_host():
    lib = spark.load()
    A = 0x7F0000000000
    rows = 8 * 32768 * 8
    # value cache: rows of 16 mask bytes + 2 bytes per kept entry, no statistic, no a section
    assert spark.packed_values_bytes(_desc(keep_v=64)) == 256 + rows * 144
    assert spark.packed_values_bytes(_desc(keep_v=26)) == 256 + rows * 72       # 68 -> rows are 8-byte multiples
    assert spark.packed_values_bytes(_desc()) == 0                               # keep_v = 0: values stay dense
    assert spark.packed_values_bytes(_desc(keep_v=129)) == 0
    d = _desc(keep_v=64)
    ok_ws = spark.decode_workspace_bytes(d)
    assert lib.spark_prune_values(ctypes.byref(_desc()), A, A, None) == 1        # keep_v missing
    assert lib.spark_prune_values(ctypes.byref(d), None, A, None) == 1
    assert lib.spark_prune_values(ctypes.byref(d), A, A + 64, None) == 1         # packed buffer misaligned
    assert lib.spark_prune_values(ctypes.byref(_desc(keep_v=64, v_token_stride=1 << 25)), A, A, None) == 2
    assert lib.spark_decode_attn_values(ctypes.byref(d), A, A, None, A, A, A, ok_ws, None) == 1
    assert lib.spark_decode_attn_values(ctypes.byref(_desc()), A, A, A, A, A, A, ok_ws, None) == 1
    assert lib.spark_unpack_values(ctypes.byref(d), None, None, None, None) == 1
    # appended rows: capacity enters the workspace size (one spare slot per 256 rows)
    dt = _desc(tail_capacity=600)
    assert spark.decode_workspace_bytes(dt) == (73 * 32 + 8 * 32 * 3) * 130 * 4 + 256
    ws_t = spark.decode_workspace_bytes(dt)
    assert lib.spark_decode_attn_tail(ctypes.byref(dt), A, A, A, A, None, A, A, A, A, ws_t, None) == 1
    assert lib.spark_decode_attn_tail(ctypes.byref(dt), A, A, A, A, A, None, A, A, A, ws_t, None) == 1
    assert lib.spark_decode_attn_tail(ctypes.byref(dt), A, A, A, A, A + 8, A, A, A, A, ws_t, None) == 1
    assert lib.spark_decode_attn_tail(ctypes.byref(_desc()), A, A, A, A, A, A, A, A, A, ws_t, None) == 1   # capacity 0
    assert lib.spark_decode_attn_tail(ctypes.byref(dt), A, A, A, A, A, A, A, A, A, ws_t - 1, None) == 3
    assert spark.packed_bytes(_desc(tail_capacity=-1)) == 0


def test_size_limits_of_the_description():
    assert spark.packed_bytes(_desc(batch=1, total_tokens=(1 << 31) - 256)) > 0
    assert spark.packed_bytes(_desc(batch=1, total_tokens=(1 << 31) - 255)) == 0
    assert spark.packed_bytes(_desc(batch=(1 << 18) + 1)) == 0


def test_statistics_rows_and_sampled_decode_arguments():
    lib = spark.load()
    A = 0x7F0000000000
    rows = 8 * 32768 * 8
    ds = _desc(stats=1)
    assert spark.packed_bytes(ds) == 256 + 2 * 8 * 8 * 128 * 4 + rows * 80      # 72 + mean + standard deviation
    # int8 storage: mask 16 + mu 4 + scale 4 + mean and standard deviation 8 + 7 code words 28 = 60 -> 64-byte rows
    assert spark.packed_bytes(_desc(stats=1, pack_dtype=spark.PACK_INT8)) == 256 + 2 * 8 * 8 * 128 * 4 + rows * 64
    assert spark.packed_bytes(_desc(stats=2)) == 0
    ws = spark.decode_workspace_bytes(ds)
    u64 = ctypes.c_uint64(1)
    assert lib.spark_decode_attn_sampled(ctypes.byref(_desc()), A, A, A, A, A, A, ws, 1, u64, None) == 1   # no stats
    assert lib.spark_decode_attn_sampled(ctypes.byref(ds), A, A, A, A, A, A, ws, 0, u64, None) == 1        # bad kind
    assert lib.spark_decode_attn_sampled(ctypes.byref(ds), A, A, A, A, A, A, ws, 3, u64, None) == 1
    assert lib.spark_decode_attn_sampled(ctypes.byref(ds), A, A, None, A, A, A, ws, 1, u64, None) == 1
    assert lib.spark_decode_attn_sampled(ctypes.byref(ds), A, A, A, A, A, A, ws - 1, 1, u64, None) == 3
    assert lib.spark_unpack_stats(ctypes.byref(_desc()), A, A, A, None) == 1
    assert lib.spark_unpack_stats(ctypes.byref(ds), None, A, A, None) == 1


def test_bench_traffic_table_names_profile_files_that_hold_the_figures():
    # every stored HBM-traffic figure of bench.py comes out of the profile summary the table names
    import bench
    assert bench.TRAFFIC_PROFILES
    for (workload, pack), rel in bench.TRAFFIC_PROFILES.items():
        assert os.path.exists(os.path.join(ROOT, rel)), rel
        nbytes, src = bench.measured_traffic(workload, pack)
        assert src == rel and nbytes is not None and nbytes > 0, (workload, pack)
    assert bench.measured_traffic("no_such_workload", "bf16") == (None, None)


def test_timeline_aid_checks_its_buffer_on_the_host():
    lib = spark.load()
    assert lib.spark_decode_timeline(None, 0) == 0                       # off
    assert lib.spark_decode_timeline(0x7F0000000004, 4096) == 1          # misaligned
    assert lib.spark_decode_timeline(0x7F0000000000, 32) == 1            # no room for one block
    assert lib.spark_decode_timeline(None, 0) == 0
