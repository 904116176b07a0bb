"""Host-side arithmetic of the carry chain's status-word tags (paper_2411_17887_amd/csrc/chain_tags.h), compiled for
the CPU with the tag period shrunk to 5 so that the tags wrap within a few calls.

What has to hold: inside one generation every call has a tag of its own; the tag field values 0 (a zero-filled word)
and the reserved "clears first" tag are never drawn; and a simulated workspace that follows the table's advice never
shows a call a status word that an EARLIER call wrote with the same tag."""
import ctypes
import os
import random
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
MOD = 5


@pytest.fixture(scope="module")
def shim(tmp_path_factory):
    so = str(tmp_path_factory.mktemp("chain_tags") / "libshim.so")
    subprocess.run(["g++", "-std=c++17", "-O1", "-fPIC", "-shared", f"-DTCUSCAN_TAG_MOD={MOD}u", "-o", so,
                    os.path.join(HERE, "chain_tags_shim.cpp")], check=True)
    L = ctypes.CDLL(so)
    ull = ctypes.c_ulonglong
    L.shim_call_id.argtypes = [ull, ctypes.POINTER(ctypes.c_uint), ctypes.POINTER(ull)]
    L.shim_table_new.restype = ctypes.c_void_p
    L.shim_table_free.argtypes = [ctypes.c_void_p]
    L.shim_needs_clear.argtypes = [ctypes.c_void_p, ull, ull, ull]
    L.shim_mark_dirty.argtypes = [ctypes.c_void_p, ull, ull]
    return L


def call_id(L, index):
    tag, gen = ctypes.c_uint(0), ctypes.c_ulonglong(0)
    L.shim_call_id(index, ctypes.byref(tag), ctypes.byref(gen))
    return tag.value, gen.value


def test_tags_go_round_and_generations_count_the_rounds(shim):
    assert shim.shim_tag_mod() == MOD
    reserved = shim.shim_clear_first_tag()
    assert reserved == (1 << 30) - 1
    seen = {}
    for i in range(4 * MOD + 3):
        tag, gen = call_id(shim, i)
        assert 1 <= tag <= MOD and tag != reserved
        assert gen == i // MOD + 1
        assert (gen, tag) not in seen                       # unique inside a generation
        seen[(gen, tag)] = i
    assert call_id(shim, 0) == (1, 1) and call_id(shim, MOD - 1) == (MOD, 1) and call_id(shim, MOD) == (1, 2)
    # a 64-bit call index: far beyond 2^32 calls the arithmetic is still the same
    big = (1 << 40) + 3
    assert call_id(shim, big) == (big % MOD + 1, big // MOD + 1)


def test_default_period_leaves_zero_and_the_reserved_tag_free():
    src = open(os.path.join(HERE, "..", "paper_2411_17887_amd", "csrc", "chain_tags.h")).read()
    assert "#define TCUSCAN_TAG_MOD ((1u << 30) - 2u)" in src      # tags 1 .. 2^30 - 2; 2^30 - 1 is the reserved one


class Table:
    def __init__(self, L):
        self.L, self.t = L, L.shim_table_new()

    def needs_clear(self, ws, nbytes, gen):
        return bool(self.L.shim_needs_clear(self.t, ws, nbytes, gen))

    def mark_dirty(self, ws, gen):
        self.L.shim_mark_dirty(self.t, ws, gen)

    def __del__(self):
        self.L.shim_table_free(self.t)


def test_first_generation_costs_nothing_and_later_ones_clear_once(shim):
    T = Table(shim)
    for _ in range(3):
        assert not T.needs_clear(0x1000, 512, 1)           # generation 1: zero-filled by its owner, nothing older exists
    assert T.needs_clear(0x1000, 512, 2)                   # first use after the tags came round
    assert not T.needs_clear(0x1000, 512, 2)
    assert not T.needs_clear(0x1000, 256, 2)               # a smaller call on the same workspace
    assert T.needs_clear(0x1000, 1024, 2)                  # more status words than were cleared
    assert not T.needs_clear(0x1000, 1024, 2)
    assert T.needs_clear(0x2000, 512, 2)                   # another workspace
    assert T.needs_clear(0x1000, 64, 4)                    # a generation skipped entirely
    assert T.needs_clear(0x1000, 1024, 4) and not T.needs_clear(0x1000, 1024, 4)


def test_dirty_marks(shim):
    T = Table(shim)
    assert not T.needs_clear(0x1000, 512, 1)
    T.mark_dirty(0x1000, 1)                                 # a segmented call left row maps there
    assert T.needs_clear(0x1000, 512, 1)                    # ... so even in generation 1 the next plain call clears
    assert not T.needs_clear(0x1000, 512, 1)
    assert not T.needs_clear(0x3000, 512, 1)                # workspaces never marked stay free of charge
    T.mark_dirty(0x1000, 1)
    T.mark_dirty(0x1000, 1)
    assert T.needs_clear(0x1000, 8, 1) and not T.needs_clear(0x1000, 8, 1)
    # more dirty workspaces than the table holds: a mark is displaced, and from then on unknown workspaces are cleared
    slots = shim.shim_slots()
    for i in range(slots + 1):
        T.mark_dirty(0x100000 + 0x1000 * i, 1)
    assert T.needs_clear(0x100000, 64, 1)                   # the displaced one
    assert T.needs_clear(0x999000, 64, 1)                   # and any workspace the table does not know


def test_simulated_workspaces_never_show_a_stale_word(shim):
    """Replays random call sequences against a model of workspace memory: words hold (tag, call index) pairs; a call
    clears if the table says so, then must not find its own tag on a word it has not written itself."""
    rng = random.Random(2411)
    for trial in range(20):
        T = Table(shim)
        n_ws = rng.choice([1, 3, 70])                       # 70: more workspaces than table slots
        memory = {w: {} for w in range(n_ws)}               # workspace -> {word index: (tag, writer)}
        index = 0
        for step in range(600):
            w = rng.randrange(n_ws)
            words = rng.choice([1, 4, 9])
            if rng.random() < 0.1:
                index += rng.randrange(3 * MOD)             # other calls elsewhere in the process draw tags too
            if rng.random() < 0.05:
                T.mark_dirty(0x1000 * (w + 1), call_id(shim, index)[1])
                for k in range(12):                         # row maps: arbitrary bits, any of them may look like a tag
                    memory[w][k] = (rng.randrange(1, MOD + 1), -1)
                continue
            tag, gen = call_id(shim, index)
            if T.needs_clear(0x1000 * (w + 1), 256 + 64 * words, gen):
                for k in range(words):
                    memory[w].pop(k, None)
            for k in range(words):
                assert memory[w].get(k, (0, None))[0] != tag, (trial, step, "stale word passes for a published one")
            for k in range(words):
                memory[w][k] = (tag, index)
            index += 1
