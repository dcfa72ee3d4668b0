"""Are the oracle's pins sharp?  Plant one plausible mistake at a time in a copy
of kv_oracle.c (a dropped term, a wrong index, transposed operands, an off-by-one,
a forgotten flag), build it, and require that at least one pin of
test_oracle_pins.py fails on it.  Everything here runs on the CPU; each mutant
runs in a child process so that a mutant that crashes only ends the child.
"""
import os
import subprocess
import sys

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(ROOT, "oracle", "kv_oracle.c")

# (name, text to find, replacement, how many places it must occur in)
MUTANTS = [
    ("kv_layer_order", "(2 * l + kv) * s->chunk", "(2 * kv + l) * s->chunk", 2),
    ("v_dropped", "kv * c->kv_stride + phys", "0 * c->kv_stride + phys", 2),
    ("layer_dropped", "c->pool + l * c->layer_stride + kv * c->kv_stride + phys",
     "c->pool + 0 * c->layer_stride + kv * c->kv_stride + phys", 2),
    ("last_byte_dropped", "for (int64_t b = 0; b < s->chunk; b++) dst[b] = src[b];",
     "for (int64_t b = 0; b + 1 < s->chunk; b++) dst[b] = src[b];", 3),
    ("scale_offset_dropped", "c->staging + slot * s->S + s->block_bytes + (2 * l + kv) * s->scale_chunk",
     "c->staging + slot * s->S + (2 * l + kv) * s->scale_chunk", 2),
    ("scale_block_index", "kv * c->s_kv_stride + phys * c->s_block_stride",
     "kv * c->s_kv_stride + 0 * c->s_block_stride", 2),
    ("wm_counts_tail_full", "nb.e[k].wm = (int32_t)(len / B);", "nb.e[k].wm = (int32_t)((len + B - 1) / B);", 1),
    ("wm_counts_tail_delta", "nb.e[k].wm = (int32_t)(m < full ? m : full);", "nb.e[k].wm = (int32_t)m;", 1),
    ("budget_ignored", "if (!unlimited && m > wm + left) m = wm + left;", ";", 1),
    ("budget_not_charged", "if (!unlimited) left -= (m - wm);", ";", 1),
    ("delta_rereads_old_blocks", "for (int64_t j = wm; j < m; j++)", "for (int64_t j = 0; j < m; j++)", 1),
    ("staged_shrinks", "if (m > nb.e[k].staged) nb.e[k].staged = (int32_t)m;", "nb.e[k].staged = (int32_t)m;", 1),
    ("first_fit_off_by_one", "s + want <= b->slots", "s + want < b->slots", 1),
    ("release_keeps_slots", "for (int64_t k = 0; k < b->e[i].cap; k++) b->used[b->e[i].base + k] = 0;", ";", 1),
    ("grow_over_neighbour", "if (b->used[e->base + k]) return ORA_ENOSPC;", ";", 1),
    ("swapped_never_set", "nb.e[k].swapped = 1;", "nb.e[k].swapped = 0;", 1),
    ("csr_offset_ignored", "moves_push(&mv, block_ids[offsets[i] + j], nb.e[k].base + j)) { rc = ORA_EINVAL; break; }\n    nb.e[k].staged",
     "moves_push(&mv, block_ids[j], nb.e[k].base + j)) { rc = ORA_EINVAL; break; }\n    nb.e[k].staged", 1),
    ("swap_in_transposed", "slot_to_block(s, mv.slot[m], mv.phys[m]);", "slot_to_block(s, mv.phys[m] % s->bk.slots, mv.slot[m]);", 1),
    ("swap_in_reads_pool", "for (int64_t m = 0; m < mv.n; m++) slot_to_block(s, mv.slot[m], mv.phys[m]);",
     "for (int64_t m = 0; m < mv.n; m++) block_to_slot(s, mv.phys[m], mv.slot[m]);", 1),
    ("dup_check_dropped", "if (mv.phys[a] == mv.phys[b]) { rc = ORA_EDUP; break; }", ";", 1),
    ("keep_flag_inverted", "if (flags & ORA_KEEP_STAGING)", "if (!(flags & ORA_KEEP_STAGING))", 1),
    ("row_length_unchecked", "if (len < 0 || row != (len + B - 1) / B) { rc = ORA_EINVAL; break; }", ";", 1),
    ("partial_effect_on_error", "  if (rc) {\n    book_free(&nb);\n    moves_free(&mv);\n    return rc;\n  }\n  book_free(&s->bk);\n  s->bk = nb;\n  for (int64_t m = 0; m < mv.n; m++) block_to_slot(s, mv.phys[m], mv.slot[m]);\n  moves_free(&mv);\n  return ORA_OK;",
     "  for (int64_t m = 0; m < mv.n; m++) block_to_slot(s, mv.phys[m], mv.slot[m]);\n  if (rc) {\n    book_free(&nb);\n    moves_free(&mv);\n    return rc;\n  }\n  book_free(&s->bk);\n  s->bk = nb;\n  moves_free(&mv);\n  return ORA_OK;", 1),
    ("move_blocks_reversed", "block_to_block(s, src_ids[i], dst_ids[i]);", "block_to_block(s, dst_ids[i], src_ids[i]);", 1),
    ("tail_ignored_by_flag", "(flags & ORA_DELTA_INCLUDE_TAIL) ? (len + B - 1) / B : full", "full", 1),
]

RUNNER = r"""
import sys
sys.path.insert(0, {root!r}); sys.path.insert(0, {here!r})
from oracle import kv_oracle as ko
import test_oracle_pins as T
lib = ko._load({lib!r})
failed = None
for fn, args in T.PINS:
    try:
        fn(*args, lib=lib)
    except AssertionError:
        failed = fn.__name__
        break
print("CAUGHT_BY", failed)
sys.exit(0 if failed else 3)
"""


def _run_pins(lib):
    code = RUNNER.format(root=ROOT, here=HERE, lib=lib)
    return subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=300)


def _build(text, out):
    src = out + ".c"
    with open(src, "w") as f:
        f.write(text)
    subprocess.check_call(["gcc", "-O1", "-std=c99", "-fPIC", "-shared", "-I", os.path.dirname(SRC), "-o", out, src])


def test_unmutated_oracle_passes_the_runner(tmp_path):
    out = str(tmp_path / "ok.so")
    _build(open(SRC).read(), out)
    r = _run_pins(out)
    assert r.returncode == 3 and "CAUGHT_BY None" in r.stdout, r.stdout + r.stderr


@pytest.mark.parametrize("name,old,new,count", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_mutant_is_caught(tmp_path, name, old, new, count):
    text = open(SRC).read()
    assert text.count(old) == count, "mutation site of %s moved: found %d" % (name, text.count(old))
    out = str(tmp_path / (name + ".so"))
    _build(text.replace(old, new), out)
    r = _run_pins(out)
    # caught = a pin's assertion failed (exit 0 from the runner) or the mutant crashed the child
    assert r.returncode != 3, "no pin notices mutant %s\n%s" % (name, r.stdout + r.stderr)
