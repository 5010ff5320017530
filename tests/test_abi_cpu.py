"""CPU-side checks: the library loads and exports everything include/ifx.h
declares; the slot bookkeeping matches a deque model; calls that need a device
fail loudly (there is no CPU fallback)."""
import collections
import os
import re

import pytest

from paper_2511_20714_amd import binding as ifx

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "ifx.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ifx_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = ifx.lib()
    names = declared_symbols()
    assert len(names) >= 20
    for name in names:
        assert hasattr(lib, name), name
    # and the binding wraps each of them under the same name
    for name in names:
        assert callable(getattr(ifx, name)), name


def test_header_is_plain_c():
    import subprocess, tempfile
    with tempfile.TemporaryDirectory() as d:
        src = os.path.join(d, "t.c")
        open(src, "w").write('#include "ifx.h"\nint main(void){return IFX_OK;}\n')
        subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), "-c", src,
                               "-o", os.path.join(d, "t.o")])


@pytest.mark.parametrize("cap", [1, 2, 7, 16])
def test_ring_matches_deque_model(cap):
    ring = ifx.ifx_ring_create(cap)
    try:
        model = collections.deque(maxlen=cap)
        slot_of = {}
        assert ifx.ifx_ring_block_ids(ring) == [-1] * cap
        for t in range(3 * cap + 5):
            assert ifx.ifx_ring_next_slot(ring) == t % cap
            slot = ifx.ifx_ring_commit(ring)
            if len(model) == cap:
                slot_of.pop(model[0])
            # a free slot, or the slot of the block that just fell out
            assert slot not in slot_of.values()
            model.append(t)
            slot_of[t] = slot
            assert ifx.ifx_ring_committed(ring) == t + 1
            assert ifx.ifx_ring_resident(ring) == len(model)
            ids = ifx.ifx_ring_block_ids(ring)
            want = [-1] * cap
            for o, s in slot_of.items():
                want[s] = o
            assert ids == want
            for i, o in enumerate(model):
                assert ifx.ifx_ring_slot_of_logical(ring, i) == slot_of[o]
            assert ifx.ifx_ring_slot_of_logical(ring, len(model)) == -1
            assert ifx.ifx_ring_slot_of_logical(ring, -1) == -1
        ifx.ifx_ring_reset(ring)
        assert ifx.ifx_ring_resident(ring) == 0 and ifx.ifx_ring_block_ids(ring) == [-1] * cap
    finally:
        ifx.ifx_ring_destroy(ring)


@pytest.mark.parametrize("in_place", [False, True])
def test_ring_grow_matches_a_growing_window_model(in_place):
    """ifx_ring_grow against a plain list model: the resident blocks keep their numbers and order;
    moved: they sit in slots 0, 1, ... oldest first right after the grow; in place: every block
    stays in the slot it had; either way the new slots are used next and only then the oldest
    block is evicted again; a slot never holds two resident blocks; slots in use are a prefix."""
    import random
    rng = random.Random(7 + in_place)
    for trial in range(40):
        cap = rng.randint(1, 5)
        ring = ifx.ifx_ring_create(cap)
        try:
            committed = []  # ordinals, all of them
            gone = 0        # how many of them are evicted
            slot_of = {}
            for step in range(80):
                if rng.random() < 0.12:
                    new_cap = cap + rng.randint(1, 4)
                    ifx.ifx_ring_grow(ring, new_cap, in_place)
                    old_cap, cap = cap, new_cap
                    resident = committed[gone:]
                    if not in_place:
                        slot_of = {o: i for i, o in enumerate(resident)}  # re-laid, oldest first
                    # the next commit takes a new slot, unless the old capacity was not full yet
                    assert ifx.ifx_ring_next_slot(ring) == len(resident)
                    with pytest.raises(ifx.IfxError):
                        ifx.ifx_ring_grow(ring, cap, in_place)
                    del old_cap
                else:
                    slot = ifx.ifx_ring_commit(ring)
                    if len(committed) - gone == cap:
                        assert slot == slot_of.pop(committed[gone])  # the oldest block's slot is the one reused
                        gone += 1
                    else:
                        assert slot == len(committed) - gone  # slots in use are a prefix
                    assert slot not in slot_of.values()
                    slot_of[len(committed)] = slot
                    committed.append(len(committed))
                resident = committed[gone:]
                assert ifx.ifx_ring_committed(ring) == len(committed)
                assert ifx.ifx_ring_resident(ring) == len(resident)
                want = [-1] * cap
                for o in resident:
                    want[slot_of[o]] = o
                assert ifx.ifx_ring_block_ids(ring) == want
                assert sorted(slot_of.values()) == list(range(len(resident)))
                for i, o in enumerate(resident):
                    assert ifx.ifx_ring_slot_of_logical(ring, i) == slot_of[o]
                assert ifx.ifx_ring_slot_of_logical(ring, len(resident)) == -1
        finally:
            ifx.ifx_ring_destroy(ring)


def test_reserve_is_checked_before_any_device_work():
    h = ifx.ifx_kv_cache_create(1, 2, 128, 128)
    try:
        lib = ifx.lib()
        assert lib.ifx_kv_cache_reserve(h, 64) == ifx.IFX_ERR_INVALID_ARG  # below the capacity
        assert lib.ifx_kv_cache_reserve(None, 256) == ifx.IFX_ERR_INVALID_ARG
        assert lib.ifx_kv_cache_reserve(h, 200) == ifx.IFX_OK
        assert lib.ifx_kv_cache_configure(h, 64, ifx.IFX_BF16, 0.0) == ifx.IFX_ERR_INVALID_ARG  # 200 % 64
    finally:
        ifx.ifx_kv_cache_destroy(h)


def test_ring_rejects_bad_capacity():
    with pytest.raises(ifx.IfxError):
        ifx.ifx_ring_create(0)


def test_create_rejects_bad_sizes():
    for args in [(0, 2, 64, 128), (1, 0, 64, 128), (1, 2, 0, 128), (1, 2, 64, 0), (1, 2, 64, -5)]:
        with pytest.raises(ifx.IfxError):
            ifx.ifx_kv_cache_create(*args)


def test_calls_before_configure_fail():
    h = ifx.ifx_kv_cache_create(2, 2, 128, 64)
    try:
        lib = ifx.lib()
        assert lib.ifx_kv_cache_len(h, 0) == ifx.IFX_ERR_NOT_CONFIGURED
        assert lib.ifx_kv_cache_commit(h, 0, 16, 16, None) == ifx.IFX_ERR_NOT_CONFIGURED
        assert lib.ifx_block_attention(h, 0, 16, 16, 16, 16, None) == ifx.IFX_ERR_NOT_CONFIGURED
        assert "configure" in ifx.ifx_last_error()
        assert lib.ifx_kv_cache_configure(h, 48, ifx.IFX_BF16, 0.0) == ifx.IFX_ERR_INVALID_ARG  # 64 % 48
        assert lib.ifx_kv_cache_configure(h, 64, 7, 0.0) == ifx.IFX_ERR_INVALID_ARG
        assert lib.ifx_kv_cache_configure(None, 64, 0, 0.0) == ifx.IFX_ERR_INVALID_ARG
    finally:
        ifx.ifx_kv_cache_destroy(h)
    ifx.ifx_kv_cache_destroy(None)


def test_no_cpu_fallback_without_a_device():
    torch = pytest.importorskip("torch")
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(ifx.IfxError) as e:
        ifx.KVCache(1, 2, 64, 1024, 256, ifx.IFX_F32)
    assert e.value.code == ifx.IFX_ERR_HIP


def test_bench_refuses_more_than_one_gpu():
    """bench.py is a one-GPU benchmark: any other --gpus value ends with a message, before any GPU work."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "one GPU" in (r.stderr + r.stdout)


def test_oracle_is_not_imported_by_the_product():
    """The package must not reach for the oracle (test infrastructure) or for working files."""
    pkg = os.path.join(ROOT, "paper_2511_20714_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hpp", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text, f
                assert "_work" not in text, f


@pytest.mark.parametrize("heads", [1, 2, 3, 5, 7, 8, 9, 11, 12, 13, 16, 17, 24, 40])
def test_attention_launch_items_tile_every_head(heads):
    """The bf16 attention launch: the workgroups' (head, query rows) items, decoded by the function
    the kernel itself uses, cover rows 0 .. n - 1 of every head exactly once, in wavefronts of 32
    rows, at most 8 per workgroup and dealt evenly (counts differ by at most one, no workgroup
    is empty unless it exits); a head's workgroups sit on as few XCDs as its share allows."""
    for n in (8, 32, 72, 200, 256, 264, 2056, 4680, 10800):
        grid = ifx.ifx_attention_launch_grid(n, heads)
        q_tiles = -(-n // 256)
        assert grid % 8 == 0 and grid >= heads * q_tiles
        covered = collections.defaultdict(list)  # head -> [(row0, waves)]
        xcds = collections.defaultdict(set)
        tiles = collections.defaultdict(set)
        for w in range(grid):
            head, q_tile, row0, waves, xcd = ifx.ifx_attention_launch_item(n, heads, w)
            assert xcd == w % 8
            if waves == 0:
                continue
            assert 0 <= head < heads and 1 <= waves <= 8 and row0 % 32 == 0
            assert q_tile not in tiles[head]
            tiles[head].add(q_tile)
            covered[head].append((row0, waves))
            xcds[head].add(xcd)
        assert sorted(covered) == list(range(heads))
        for head, items in covered.items():
            items.sort()
            assert len(items) == q_tiles
            nxt = 0
            for row0, waves in items:
                assert row0 == nxt, (n, heads, head)
                nxt = row0 + 32 * waves
            assert n <= nxt < n + 32  # the last wavefront holds the last row
            counts = [wv for _, wv in items]
            assert max(counts) - min(counts) <= 1
        # whole heads live on one XCD each, eight at a time; the rest on as few as an even split needs
        left = heads % 8
        for head in range(heads):
            if head < heads - left:
                assert len(xcds[head]) == 1
            elif 8 % left == 0:
                assert len(xcds[head]) <= 8 // left


def test_attention_launch_shape_rejects_bad_arguments():
    with pytest.raises(ifx.IfxError):
        ifx.ifx_attention_launch_grid(0, 12)
    with pytest.raises(ifx.IfxError):
        ifx.ifx_attention_launch_grid(4680, 0)
    grid = ifx.ifx_attention_launch_grid(4680, 12)
    assert grid == 232  # 8 x (19 workgroups of a whole head + 10 of a shared one); 228 of them have rows
    with pytest.raises(ifx.IfxError):
        ifx.ifx_attention_launch_item(4680, 12, grid)
    with pytest.raises(ifx.IfxError):
        ifx.ifx_attention_launch_item(4680, 12, -1)
    busy = [ifx.ifx_attention_launch_item(4680, 12, w) for w in range(grid)]
    assert sum(1 for it in busy if it[3] > 0) == 228
    assert sorted(it[3] for it in busy if it[0] == 0 and it[3] > 0) == [7] * 5 + [8] * 14
