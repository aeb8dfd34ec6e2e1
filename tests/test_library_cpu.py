"""CPU-side checks of the C-ABI library: it loads, exports every declared symbol, sizes its
workspaces sanely and rejects bad arguments on the host (no kernel is launched here)."""
import ctypes
import os
import re

import pytest

import paper_2404_11912_amd as tf
from paper_2404_11912_amd.binding import tf_kv_desc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "triforce.h")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(tf.LIB_PATH):
        from paper_2404_11912_amd.build import build_library
        build_library()
    return tf.load_library()


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tf_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared_functions()
    assert set(names) == set(tf.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_version_and_status_strings(lib):
    assert tf.tf_version() >= 100
    for code in (0, -1, -2, -3, -4, -99):
        assert lib.tf_status_string(code)


def test_workspace_queries(lib):
    full = tf.tf_decode_attn_full_workspace_bytes(1, 32, 131072, 5)
    retr = tf.tf_decode_attn_retrieval_workspace_bytes(1, 32, 4096, 3)
    assert 0 < retr <= full < 64 << 20                 # partials stay far below the 2 GiB of KV per layer
    assert tf.tf_chunk_topk_gather_workspace_bytes(1, 32, 16384, 512) >= 32 * 16384 * 4
    seg = 8                                            # 32000 entries in segments of 4096
    assert tf.tf_spec_accept_workspace_bytes(4, 5, 32000) == (4 * 9 * seg * 4 + 4 * seg * 1024 + 4 * seg) * 8
    assert tf.tf_decode_attn_full_workspace_bytes(0, 32, 10, 1) == 0


def _nsplit(kind, B, H, N):
    return tf.tf_decode_attn_plan(kind, B, H, N)[0]


def test_split_planning(lib):
    """Without a GPU the planner assumes 256 CUs. Long caches whose units divide the CU count get
    one workgroup per CU; others get equal splits on a whole number of workgroups per CU."""
    full, retr, indexed = 0, 1, 2
    assert tf.tf_decode_attn_plan(full, 1, 32, 131072) == (8, 16384)
    assert _nsplit(full, 1, 32, 1048576) == 8
    assert _nsplit(full, 4, 32, 65536) == 2
    assert _nsplit(full, 2, 32, 57344) == 4
    assert _nsplit(full, 6, 32, 19456) == 4                         # 768 workgroups: three per CU
    assert _nsplit(full, 10, 32, 12288) == 4
    assert _nsplit(retr, 1, 32, 4096) == 8
    assert _nsplit(full, 1, 1, 3) == 1                              # never more splits than 512-token pieces
    assert _nsplit(full, 1, 4, 4096) == 8
    assert _nsplit(full, 1, 1, 1 << 30) <= 2048                     # the merge kernel's limit
    assert _nsplit(indexed, 1, 32, 512 * 8 + 3) == 24


def test_workspace_queries_are_monotone_in_the_length(lib):
    """The planned split count snaps to counts that fill the CUs evenly, so it is not monotone in
    the length (4096 tokens of 32 units plan more splits than 4100); the workspace query sizes for
    the most splits any shorter length could plan, so a workspace queried for a bound serves
    every call below it."""
    per_split = 4 * (8 * 128 + 16) * 4               # one partial per wave: 8 rows x (128 + 2) floats each
    for kind, query in ((0, tf.tf_decode_attn_full_workspace_bytes), (1, tf.tf_decode_attn_retrieval_workspace_bytes)):
        for BH in (1, 4, 32, 192):
            prev = 0
            for n in list(range(1, 300, 7)) + list(range(3900, 4400, 9)) + [8192, 65536, 131072]:
                ws = query(1, BH, n, 5)
                assert ws >= prev
                prev = ws
                assert ws >= BH * _nsplit(kind, 1, BH, n) * per_split
    q = tf.tf_decode_attn_indexed_workspace_bytes
    assert q(1, 32, 512, 8, 64, 3) >= 32 * max(_nsplit(2, 1, 32, 512 * 8 + r) for r in range(0, 65)) * per_split


def test_options(lib):
    tf.tf_set_option("attn_full_tokens_per_split", 256)
    small = tf.tf_decode_attn_full_workspace_bytes(1, 1, 4096, 4)
    plan = tf.tf_decode_attn_plan(0, 1, 1, 4096)
    tf.tf_set_option("attn_full_tokens_per_split", 0)
    assert small == 16 * 4 * (8 * 128 + 16) * 4 and plan == (16, 256)
    with pytest.raises(tf.TfError):
        tf.tf_set_option("attn_full_tokens_per_split", 100)      # not a multiple of 64
    with pytest.raises(tf.TfError):
        tf.tf_set_option("no_such_option", 1)


def test_thread_options_are_private_to_their_thread(lib):
    """A knob set with tf_set_thread_option is seen by the setting thread only; other threads keep
    the process-wide value; -1 removes the override."""
    import threading
    seen = {}

    def worker(name, tps):
        if tps is not None:
            tf.tf_set_thread_option("attn_full_tokens_per_split", tps)
        barrier.wait(timeout=30)                    # all overrides are in place before anyone plans
        seen[name] = tf.tf_decode_attn_plan(0, 1, 1, 8192)
        if tps is not None:
            tf.tf_set_thread_option("attn_full_tokens_per_split", -1)
            seen[name + "_after"] = tf.tf_decode_attn_plan(0, 1, 1, 8192)

    barrier = threading.Barrier(3)
    auto = tf.tf_decode_attn_plan(0, 1, 1, 8192)
    ts = [threading.Thread(target=worker, args=a) for a in (("a", 256), ("b", 1024), ("c", None))]
    for t in ts:
        t.start()
    for t in ts:
        t.join()
    assert seen["a"] == (32, 256) and seen["b"] == (8, 1024) and seen["c"] == auto
    assert seen["a_after"] == auto and seen["b_after"] == auto
    assert tf.tf_decode_attn_plan(0, 1, 1, 8192) == auto
    with pytest.raises(tf.TfError):
        tf.tf_set_thread_option("attn_full_tokens_per_split", 100)


def test_host_side_argument_checks(lib):
    """Every call validates on the host and returns before touching the GPU."""
    d = tf_kv_desc(1, 2, 128, 0, 64, 2 * 64 * 128, 64 * 128, 128)
    bad_dim = tf_kv_desc(1, 2, 96, 0, 64, 2 * 64 * 96, 64 * 96, 96)
    d64 = tf_kv_desc(1, 2, 64, 0, 64, 2 * 64 * 64, 64 * 64, 64)        # attention and append only
    p = ctypes.c_void_p(4096)          # never dereferenced on the host
    ref = ctypes.byref
    # null pointers
    assert lib.tf_decode_attn_full(None, p, p, ref(d), None, 64, 4, 1.0, 1, p, None, p, 1 << 20, None) == -1
    assert lib.tf_chunk_summarize(None, ref(d), 8, 0, 8, p, 8, None) == -1
    assert lib.tf_spec_accept(None, p, p, 1, 2, 10, 1.0, p, p, p, p, p, 1 << 10, None) == -1
    assert lib.tf_decode_attn_tree(p, p, p, ref(d), None, 64, 4, 1.0, None, p, None, p, 1 << 20, None) == -1
    m4 = (ctypes.c_uint16 * 4)(1, 3, 5, 9)
    assert lib.tf_decode_attn_tree(p, p, p, ref(d), None, 3, 4, 1.0, m4, p, None, p, 1 << 20, None) == -1   # fewer rows than G
    assert lib.tf_decode_attn_tree(p, p, p, ref(d), None, 64, 4, 1.0, m4, p, None, p, 16, None) == -3
    assert lib.tf_spec_accept_ragged(p, p, p, None, 1, 2, 10, 1.0, p, p, p, p, p, 1 << 20, None) == -1
    # unsupported shapes
    assert lib.tf_decode_attn_full(p, p, p, ref(bad_dim), None, 64, 4, 1.0, 1, p, None, p, 1 << 20, None) == -2
    assert lib.tf_decode_attn_full(p, p, p, ref(d), None, 64, 17, 1.0, 1, p, None, p, 1 << 20, None) == -2
    m17 = (ctypes.c_uint16 * 17)(*([1] * 17))
    assert lib.tf_decode_attn_tree(p, p, p, ref(d), None, 64, 17, 1.0, m17, p, None, p, 1 << 20, None) == -2
    assert lib.tf_chunk_summarize(p, ref(d64), 8, 0, 8, p, 8, None) == -2
    assert lib.tf_decode_attn_full(p, p, p, ref(d64), None, 64, 4, 1.0, 1, p, None, p, 16, None) == -3   # accepted up to the workspace check
    assert lib.tf_chunk_topk_gather(p, p, 8, p, p, ref(d), 8, None, 8, 4096, p, None, None, None, None,
                                    p, 1 << 20, None) == -2
    # inconsistent sizes
    assert lib.tf_decode_attn_full(p, p, p, ref(d), None, 65, 4, 1.0, 1, p, None, p, 1 << 20, None) == -1
    assert lib.tf_decode_attn_full(p, p, p, ref(d), None, 3, 4, 1.0, 1, p, None, p, 1 << 20, None) == -1
    assert lib.tf_chunk_summarize(p, ref(d), 8, 0, 9, p, 16, None) == -1       # 9 chunks of 8 > capacity 64
    assert lib.tf_chunk_topk_gather(p, p, 8, p, p, ref(d), 8, None, 8, 9, p, None, None, None, None,
                                    p, 1 << 20, None) == -1                    # k > n_chunks
    assert lib.tf_spec_accept(p, p, p, 1, 2, 10, -1.0, p, p, p, p, p, 1 << 10, None) == -1
    # workspace too small / missing
    assert lib.tf_decode_attn_full(p, p, p, ref(d), None, 64, 4, 1.0, 1, p, None, p, 16, None) == -3
    assert lib.tf_decode_attn_retrieval(p, p, p, ref(d), None, 64, 4, 1.0, 1, p, None, None, 0, None) == -3
    assert lib.tf_spec_accept(p, p, p, 1, 2, 10, 1.0, p, p, p, p, p, 8, None) == -3
    # empty range is a no-op that succeeds
    assert lib.tf_chunk_summarize(p, ref(d), 8, 0, 0, p, 8, None) == 0


def test_binding_refuses_cpu_tensors():
    import torch
    x = torch.zeros(1, 1, 16, 128, dtype=torch.bfloat16)
    with pytest.raises(TypeError):
        tf.kv_desc(x)


def test_header_is_valid_c99_and_cxx():
    """include/triforce.h must compile on its own as C99 and as C++ (no HIP or torch types in it)."""
    import subprocess
    import tempfile
    inc = os.path.dirname(HEADER)
    for lang, std in (("c", "-std=c99"), ("c++", "-std=c++11")):
        with tempfile.NamedTemporaryFile("w", suffix=".c" if lang == "c" else ".cc") as f:
            f.write('#include "triforce.h"\nint main(void) { tf_kv_desc d; d.q_group = 0; return d.q_group + TF_OK; }\n')
            f.flush()
            subprocess.check_call(["gcc" if lang == "c" else "g++", std, "-Wall", "-Werror", "-pedantic", "-fsyntax-only",
                                   "-I", inc, f.name])
