"""Host-only checks: the library loads and exports the whole C ABI, configuration errors are reported
without a GPU, and the chunk schedule matches its plain-Python statement."""
import os
import re

import numpy as np
import pytest

from oracle import partition_ref
from paper_2604_23838_amd import binding as jb
from paper_2604_23838_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.parametrize("header,names", [("jigsaw_decode.h", jb.EXPORTS), ("jigsaw_decode_bench.h", jb.BENCH_EXPORTS)])
def test_every_declared_symbol_is_exported(header, names):
    text = open(os.path.join(ROOT, "include", header)).read()
    declared = set(re.findall(r"\b(jd_[a-z_]+)\s*\(", text))
    assert declared, "no declarations found"
    assert declared == set(names)
    lib = jb.lib()
    for name in declared:
        assert hasattr(lib, name), name


def test_product_header_holds_no_inspection_calls():
    text = open(os.path.join(ROOT, "include", "jigsaw_decode.h")).read()
    assert "jd_debug" not in text and "jd_bench" not in text and "jigsaw_decode_bench.h" not in text


def good_config():
    return jb.jd_config(4, 8, 2, 64, 16, 63, 100, 0.0, 0)


def test_config_validation_without_gpu():
    assert jb.jd_validate_config(good_config()) == jb.JD_OK
    assert jb.jd_workspace_bytes(good_config()) > 0
    bad = [("head_dim", 96, jb.JD_ERR_UNSUPPORTED), ("page_size", 32, jb.JD_ERR_UNSUPPORTED),
           ("num_kv_heads", 3, jb.JD_ERR_INVALID_ARG), ("batch", 0, jb.JD_ERR_INVALID_ARG),
           ("num_pages", -1, jb.JD_ERR_INVALID_ARG), ("max_pages_per_seq", 0, jb.JD_ERR_INVALID_ARG),
           ("batch", 8193, jb.JD_ERR_UNSUPPORTED), ("cu_budget", -2, jb.JD_ERR_INVALID_ARG),
           ("softmax_scale", float("nan"), jb.JD_ERR_INVALID_ARG), ("softmax_scale", -1.0, jb.JD_ERR_INVALID_ARG)]
    for field, value, want in bad:
        c = good_config()
        setattr(c, field, value)
        assert jb.jd_validate_config(c) == want, field
        assert jb.jd_last_error_string() != "no error"
        assert jb.jd_workspace_bytes(c) == 0
        with pytest.raises(jb.JdError) as e:   # rejected before any GPU call
            jb.jd_create(c)
        assert e.value.status == want
    c = good_config()
    c.num_q_heads, c.num_kv_heads = 34, 2      # group of 17 rows does not fit a 16-row tile
    assert jb.jd_validate_config(c) == jb.JD_ERR_UNSUPPORTED
    c = good_config()
    c.num_q_heads, c.num_kv_heads = 6, 2      # any group size up to 16 is served, powers of two or not
    assert jb.jd_validate_config(c) == jb.JD_OK
    c = good_config()
    c.batch, c.max_pages_per_seq, c.num_kv_heads, c.num_q_heads = 1 << 20, 1 << 10, 8, 8
    assert jb.jd_validate_config(c) == jb.JD_ERR_INVALID_ARG


def test_null_handle_and_pointer_errors_without_gpu():
    lib = jb.lib()
    assert lib.jd_decode_attention(None, 1, 1, 1, 1, 1, 1, None) == jb.JD_ERR_INVALID_ARG
    assert lib.jd_prefill_attention(None, 1, 1, 1, 1, 1, 1, 1, 16, 16, 1, None) == jb.JD_ERR_INVALID_ARG
    assert lib.jd_decode_attention_static(None, 1, 1, 1, 1, 1, 1, None) == jb.JD_ERR_INVALID_ARG
    import ctypes
    assert lib.jd_decode_attention_static(ctypes.byref(good_config()), 16, 16, None, 16, 16, 16, None) == jb.JD_ERR_INVALID_ARG
    assert lib.jd_append_kv(None, 1, 1, 1, 1, 1, 1, None, None) == jb.JD_ERR_INVALID_ARG
    assert lib.jd_check_device_flags(None, None) == jb.JD_ERR_INVALID_ARG
    assert lib.jd_debug_partition(None, None, None, None, None, None) == jb.JD_ERR_INVALID_ARG
    assert lib.jd_bench_decode_attention_vector(None, 1, 1, 1, 1, 1, 1, None) == jb.JD_ERR_INVALID_ARG
    assert lib.jd_destroy(None) == jb.JD_OK
    assert lib.jd_wave_slots(None) == 0
    assert lib.jd_debug_stream_read(None, 16, None, None) == jb.JD_ERR_INVALID_ARG
    assert lib.jd_debug_stream_copy(None, None, 16, None) == jb.JD_ERR_INVALID_ARG


def test_schedule_is_valid():
    # what fixes the schedule is validity: the active groups cover the line, none is empty, none beyond the slots
    rng = np.random.default_rng(0)
    cases = [(0, 1024), (1, 1024), (4095, 1024), (4096, 1024), (4097, 1024), (478_616, 1024), (87_736, 1024),
             (2_000_000_000, 4096), (500, 4)]
    cases += [(int(u), int(s)) for u, s in zip(rng.integers(0, 5_000_000, 200), rng.choice([4, 28, 1024, 2048], 200))]
    for units, slots in cases:
        span, active = jb.jd_debug_schedule(units, slots)
        assert span >= 1 and 0 <= active <= slots, (units, slots)
        assert (active - 1) * span < units <= active * span or (units == 0 and active == 0), (units, slots)


@pytest.mark.parametrize("wg,hkv", [(1, 2), (2, 2), (4, 8), (8, 8), (1, 5)])
def test_reference_partition_covers_every_page_once(wg, hkv):
    rng = np.random.default_rng(1)
    lens = np.floor(rng.lognormal(np.log(700.0), 1.2, size=300)).astype(int).clip(0, 9000)
    lens[::17] = 0
    slots, maxp = 64, 2048
    hdr, starts, cum = partition_ref.partition(lens, hkv, slots, maxp, group_waves=wg)
    segs = partition_ref.segments(lens, hkv, slots, maxp, group_waves=wg)
    seen = {}
    for w, b, kv, p0, p1 in segs:
        assert p1 > p0 and kv % wg == w % wg
        for pg in range(p0, p1):
            assert (b, kv, pg) not in seen
            seen[(b, kv, pg)] = w
    assert len(seen) == hdr[0] * wg == sum(partition_ref.pages(int(L), maxp) for L in lens) * hkv
    # every wave gets the same number of pages (the waves of the last group the remainder), in line order
    nwaves = hdr[2] * wg
    units = np.zeros(nwaves, dtype=int)
    for w, b, kv, p0, p1 in segs:
        units[w] += p1 - p0
    assert (units[:-wg] == hdr[1]).all() and (units[-wg:] == units[-1]).all() and 0 < units[-1] <= hdr[1]
    # the first segment of every wave is where wave_start says it begins
    first = {}
    for w, b, kv, p0, _ in segs:
        first.setdefault(w, [b, kv, p0, 0])
    assert [first[w] for w in range(nwaves)] == starts


@pytest.mark.parametrize("wg,hkv,slots", [(8, 8, 768), (8, 8, 1024), (4, 8, 100), (2, 2, 832), (1, 5, 1024), (1, 1, 28)])
def test_two_level_merge_records_never_collide(wg, hkv, slots):
    """The rule of the two-level merge, stated here in plain Python and checked on the host model of the partition:
    a sequence of one kv head that is longer than 15 spans is merged cluster by cluster (8 consecutive wave groups)
    into record ((cluster * wg + member) * 2 + side), side 0 if the sequence began before the cluster, and the
    library sets aside 2 * (slots // 8) + 16 such records.  Every (sequence, cluster) pair must get a record of
    its own below that bound, and such a sequence must reach into a second cluster."""
    cluster, flat = 8, 16
    rng = np.random.default_rng(wg * 100 + hkv)
    for trial in range(12):
        B = int(rng.integers(1, 9))
        lens = np.where(rng.random(B) < 0.6, rng.integers(6000, 70000, size=B), rng.integers(0, 300, size=B))
        maxp = 5000
        hdr, _, _ = partition_ref.partition(lens, hkv, slots, maxp, group_waves=wg)
        span = hdr[1]
        groups_of = {}
        for w, b, kv, p0, p1 in partition_ref.segments(lens, hkv, slots, maxp, group_waves=wg):
            groups_of.setdefault((b, kv), []).append(w // wg)
        used = {}
        for (b, kv), gs in groups_of.items():
            n = partition_ref.pages(int(lens[b]), maxp)
            if n <= (flat - 1) * span:
                continue
            assert gs == list(range(gs[0], gs[-1] + 1)) and len(gs) >= flat
            w0, member = gs[0], kv % wg
            clusters = sorted({g // cluster for g in gs})
            assert len(clusters) >= 2
            for c in clusters:
                rec = (c * wg + member) * 2 + (0 if w0 < c * cluster else 1)
                assert 0 <= rec < 2 * (slots // cluster) + 16, (rec, slots)
                assert rec not in used, (rec, (b, kv), used[rec])
                used[rec] = (b, kv)


def test_generator_matches_documented_totals():
    # totals of the benchmark recipe (seed 0): a change of the generator would silently move the benchmark
    want = {2: 957_219, 3: 175_455, 4: 810_848, 5: 1_738_022}
    for cfg, total in want.items():
        lens = W.draw_seq_lens(cfg, np.random.default_rng(0))
        assert int(lens.sum()) == total
    w = W.gen_config(1, 0)
    assert w.total_tokens == 1367 and w.kv_bytes == 1367 * 2 * 2 * 64 * 2
    assert w.block_table.min() == -1 and len(set(w.block_table[w.block_table >= 0].tolist())) == (w.block_table >= 0).sum()


def test_header_compiles_as_c99_and_links_from_plain_c(tmp_path):
    # the boundary is a C ABI: a C99 translation unit includes the header, links the library and calls it
    import os
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    libdir = os.path.join(root, "paper_2604_23838_amd")
    if not os.path.exists(os.path.join(libdir, "libjigsaw_decode.so")):
        pytest.skip("library not built")
    src = tmp_path / "use.c"
    src.write_text(r'''
#include "jigsaw_decode.h"
#include <stdio.h>
int main(void) {
    jd_config c = {0};
    c.batch = 4; c.num_q_heads = 8; c.num_kv_heads = 2; c.head_dim = 64; c.page_size = 16;
    c.max_pages_per_seq = 8; c.num_pages = 64;
    if (jd_validate_config(&c) != JD_OK || jd_workspace_bytes(&c) <= 0) return 1;
    c.head_dim = 96;
    if (jd_validate_config(&c) != JD_ERR_UNSUPPORTED) return 2;
    if (jd_decode_attention(0, 0, 0, 0, 0, 0, 0, 0) != JD_ERR_INVALID_ARG) return 3;
    if (jd_prefill_attention(0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0) != JD_ERR_INVALID_ARG) return 4;
    puts(jd_last_error_string(0));
    return 0;
}
''')
    exe = tmp_path / "use"
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(root, "include"),
                           str(src), "-o", str(exe), "-L", libdir, "-ljigsaw_decode", f"-Wl,-rpath,{libdir}"])
    out = subprocess.run([str(exe)], capture_output=True, text=True)
    assert out.returncode == 0, out.stdout + out.stderr
    assert "NULL" in out.stdout
