"""Mutation check of the oracle's pins (CPU only, no HIP code involved).

Each entry plants one plausible mistake in a private copy of oracle/slicer_ref.c (a dropped term, a
wrong sign or index, a different rounding, another reading of an ambiguous passage), rebuilds the copy
and runs tests/test_oracle_pins.py against it in a child process.  Every mutant must make a pin fail:
a survivor means that part of the oracle is not pinned by anything but itself.
"""
import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor


ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

# (name, text in slicer_ref.c, replacement); the text must occur in the file
MUTANTS = [
    ("tie_to_higher_index", "return a->idx < b->idx ? -1 : 1;", "return a->idx > b->idx ? -1 : 1;"),
    ("zeros_are_sent", "if (sel[r].key == 0) continue;", ";"),
    ("remainder_to_first_block", "uint32_t cnt = (m < Ms - 1) ? K : n - start;",
     "uint32_t cnt = (m > 0) ? K : n - K * (uint32_t)(Ms - 1);"),
    ("round_half_up_codes", "float r = rintf(y);", "float r = floorf(y + 0.5f);"),
    ("ceil_codes", "float r = rintf(y);", "float r = ceilf(y);"),
    ("msb_first_packing", "if ((v >> i) & 1u) bw->words", "if ((v >> (nbits - 1 - i)) & 1u) bw->words"),
    ("residual_scale", "(double)S * 0x1p-30", "(double)S * 0x1p-31"),
    ("energy_scale", "2 * e - 40", "2 * e - 41"),
    ("sign_classes_swapped", "if (neg == s) cls[n++] = sel[r];", "if (neg != s) cls[n++] = sel[r];"),
    ("largest_feasible_bitwidth", "if (chosen >= 0 && !out->s_int) break;", ";\n        if (chosen >= 0) chosen = -1;"),
    ("index_width_off_by_one", "while (((int64_t)1 << w) < N) ++w;", "while (((int64_t)1 << w) <= N) ++w;"),
    ("keep_count_ceil", "return (int64_t)floor(keep * (double)N);", "return (int64_t)ceil(keep * (double)N);"),
    ("decode_fused_multiply_add", "float a = vmin + prod;", "float a = fmaf((float)c, o, vmin);"),
    ("vmax_in_meta", "out->vmax[b] = vmax;", "out->vmax[b] = vmin;"),
    ("step_over_levels_plus_one", "o = rng / L;", "o = rng / (L + 1.0f);"),
    ("decode_step", "float o = (vmax - vmin) / L;", "float o = (vmax - vmin) / (L + 1.0f);"),
    ("row_offsets_inclusive", "put_u64(mt + off_rowoff(R, B2) + 8 * (size_t)r, total);",
     "put_u64(mt + off_rowoff(R, B2) + 8 * (size_t)r, total + seg_words[r]);"),
    ("block_minimum_dropped", "if (a < vmin) vmin = a;", ";"),
    ("always_feasible", "feasible = lhs <= rhs;", "feasible = 1;"),
    # the four that an earlier set of pins let through
    ("bf16_round_half_up", "u += 0x7FFFu + lsb;", "u += 0x8000u; (void)lsb;"),
    ("bf16_truncate", "u += 0x7FFFu + lsb;", "(void)lsb;"),
    ("reciprocal_of_step", "L / rng1;", "1.0f / (rng1 / L);"),
    ("tau_plus_in_double", "strict[r] = neg ? (a > tau_neg) : (a > tau_pos);",
     "strict[r] = neg ? (a > tau_neg) : ((double)a > (double)one_plus * (double)tau); (void)tau_pos;"),
    ("tiny_range_collapses", "int degenerate = !(rng > 0.0f);", "int degenerate = !(rng >= 0x1p-100f);"),
    ("range_not_rescaled", "float y = ldexpf(a - vmin, -er) * inv;", "float y = (a - vmin) * ldexpf(inv, -er);"),
    ("ds_floor_dropped", "uint32_t ref = c0[j] >> (qbit - q);", "uint32_t ref = (c0[j] + (1u << (qbit - q)) / 2) >> (qbit - q);"),
    ("ds_not_greedy", "if ((double)D <= delta * (double)cnt) chosen = q; else break;",
     "if ((double)D <= delta * (double)cnt) chosen = q;"),
    ("csr_pointers_inclusive", "for (int64_t row = 0; row < n_rows; ++row) { put_bits(&bw, acc, wp); acc += per_row[row]; }",
     "for (int64_t row = 0; row < n_rows; ++row) { acc += per_row[row]; put_bits(&bw, acc, wp); }"),
    ("csr_column_is_row", "put_bits(&bw, scratch_idx[j] % (uint32_t)n_cols, wc);", "put_bits(&bw, scratch_idx[j] / (uint32_t)n_cols, wc);"),
    ("csr_decode_row_off_by_one", "get_bits(rw, ppos + (uint64_t)(trow + 1) * wp, wp) <= j", "get_bits(rw, ppos + (uint64_t)(trow + 1) * wp, wp) < j"),
    ("fill_takes_from_above_tau", "else if (fill > 0 && all[r].key <= all[k - 1].key)", "else if (fill > 0)"),
]


def _run_mutant(args):
    name, old, new, base = args
    d = os.path.join(base, name)
    os.makedirs(os.path.join(d, "paper_2511_11608_amd"))
    shutil.copytree(os.path.join(ROOT, "oracle"), os.path.join(d, "oracle"),
                    ignore=shutil.ignore_patterns("*.so", "__pycache__"))
    os.makedirs(os.path.join(d, "tests"))
    for f in ("__init__.py", "conftest.py", "streamfmt.py", "test_oracle_pins.py"):
        shutil.copy(os.path.join(ROOT, "tests", f), os.path.join(d, "tests", f))
    shutil.copytree(os.path.join(ROOT, "tests", "golden"), os.path.join(d, "tests", "golden"))
    for f in ("__init__.py", "synth.py"):
        shutil.copy(os.path.join(ROOT, "paper_2511_11608_amd", f), os.path.join(d, "paper_2511_11608_amd", f))
    src = os.path.join(d, "oracle", "slicer_ref.c")
    text = open(src).read()
    if old not in text:
        return name, "mutation text not found in slicer_ref.c"
    open(src, "w").write(text.replace(old, new))
    env = dict(os.environ, PYTHONPATH=d, OMP_NUM_THREADS="1")
    p = subprocess.run([sys.executable, "-m", "pytest", "tests/test_oracle_pins.py", "-x", "-q", "-p", "no:cacheprovider"],
                       cwd=d, env=env, capture_output=True, text=True, timeout=600)
    if p.returncode == 0:
        return name, "SURVIVED: no pin fails with this mistake planted"
    if " failed" not in p.stdout:
        return name, "did not run: " + (p.stdout + p.stderr)[-400:]
    return name, None


def test_every_planted_mistake_fails_a_pin(tmp_path):
    jobs = [(n, o, r, str(tmp_path)) for n, o, r in MUTANTS]
    with ThreadPoolExecutor(max_workers=4) as ex:
        results = list(ex.map(_run_mutant, jobs))
    bad = [f"{n}: {msg}" for n, msg in results if msg]
    assert not bad, "\n".join(bad)
