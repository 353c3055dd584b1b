"""The pins are sharp: a mistake planted in a COPY of the oracle (never in the GPU path) makes
the pin named beside it fail.  Each entry replaces one piece of the C source, the copy is built
with the oracle's own flags into a temporary folder, and the pin runs in a child process that
loads the copy instead of the real library."""
import concurrent.futures
import os
import subprocess
import sys

import pytest

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PINS = "tests/test_oracle_pins.py::"
GATHER = "tests/test_gather_reduce.py::"
SEGMENT = "tests/test_segment.py::"

# (name, text in chunk_oracle.c, replacement, replace every occurrence?, pin that must fail)
MISTAKES = [
    ("duplicate applied again", "if (seen[d->seq]) continue; /* a retransmitted copy", "; /* a retransmitted copy", False,
     PINS + "test_exactly_once_all_ones"),
    ("nothing forwarded", "if (fwd) o[i] = t;", ";", True, PINS + "test_closed_loop_small_integers_exact"),
    ("accumulator not written", "if (keep) a[i] = t;", "if (keep) ;", False, PINS + "test_exactly_once_all_ones"),
    ("bf16 truncates", "return (uint16_t)((u + 0x7FFFu + lsb) >> 16);", "return (uint16_t)(u >> 16);", False,
     PINS + "test_bf16_rounding_is_nearest_even_exact"),
    ("bf16 rounds half up", "uint32_t lsb = (u >> 16) & 1u;", "uint32_t lsb = 1u;", False,
     PINS + "test_bf16_rounding_is_nearest_even_exact"),
    ("max is min", "case ORC_MAX: return (r > a) ? r : a;", "case ORC_MAX: return (r < a) ? r : a;", True,
     PINS + "test_textbook_ring_itself"),
    ("ring: wrong reduce-scatter segment", "(r + 2 * R - s - 1) % R", "(r + 2 * R - s) % R", False,
     PINS + "test_closed_loop_matches_textbook_ring"),
    ("ring: wrong allgather segment", ": (r + R - s) % R;", ": (r + R - s + 1) % R;", False,
     PINS + "test_closed_loop_matches_textbook_ring"),
    ("sum subtracts", "case ORC_SUM: return a + r;", "case ORC_SUM: return a - r;", False,
     PINS + "test_exactly_once_all_ones"),
    ("bf16 sum not rounded", "case ORC_SUM: return orc_f32_to_bf16(fa + fr);",
     "case ORC_SUM: return (uint16_t)(f32_bits(fa + fr) >> 16);", False, PINS + "test_bf16_golden_ties"),
    ("scatter applies duplicates", "    if (seen[d->seq]) continue;\n", "    ;\n", True,
     PINS + "test_alltoall_is_concatenation_of_sources"),
    ("bitmap bit order", "words[s >> 5] |= (uint32_t)1 << (s & 31);", "words[s >> 5] |= (uint32_t)1 << (31 - (s & 31));",
     False, PINS + "test_exactly_once_all_ones"),
    ("forwards the received value", "if (fwd) o[i] = t;", "if (fwd) o[i] = r[i];", True,
     PINS + "test_closed_loop_small_integers_exact"),
    ("staging offset taken from dst", "(char*)out_stage + out_at", "(char*)out_stage + (d->dst_off % 64)", True,
     PINS + "test_interleaving_invariance"),
    ("forward-only writes back", "const int keep = !(fwd && (d->out_off & ORC_FORWARD_ONLY));", "const int keep = 1;", True,
     PINS + "test_forward_only_records_relay_without_write_back"),
    ("forward-only flag left in the address", "const uint64_t out_at = d->out_off & ~ORC_FORWARD_ONLY;",
     "const uint64_t out_at = d->out_off;", True, PINS + "test_forward_only_records_relay_without_write_back"),
    ("binary16 truncates", "if (rem > 0x1000u || (rem == 0x1000u && (h & 1u))) ++h;", ";", False,
     PINS + "test_f16_conversions_against_numpy"),
    ("binary16 subnormal rounds half up", "if (rem > half || (rem == half && (h & 1u))) ++h;", "if (rem >= half) ++h;", False,
     PINS + "test_f16_conversions_against_numpy"),
    ("binary16 underflow cut one binade early", "if (e < -25) return sign;", "if (e < -24) return sign;", False,
     PINS + "test_f16_conversions_against_numpy"),
    ("int32 compared unsigned", "int32_t orc_combine_i32(int32_t a, int32_t r, int op) {",
     "int32_t orc_combine_i32(int32_t a0, int32_t r0, int op) { uint32_t a = a0, r = r0;", False,
     PINS + "test_f16_i32_f32_ops_against_numpy"),
    ("product adds", "case ORC_PROD: return a * r;", "case ORC_PROD: return a + r;", False,
     PINS + "test_f16_i32_f32_ops_against_numpy"),
    ("multi-source fold rounds per hop", "f = op == ORC_SUM ? f + fr : f * fr;",
     "f = op == ORC_SUM ? f + fr : f * fr; f = bf16_widen(orc_f32_to_bf16(f));", False,
     GATHER + "test_bf16_accumulates_in_fp32_and_rounds_once"),
    ("multi-source fold skips the last source", "for (uint32_t j = 0; j < d->n_src; ++j)",
     "for (uint32_t j = 0; j + 1 < d->n_src; ++j)", True, GATHER + "test_fp32_fold_in_listed_order_against_numpy"),
    ("message window: count not clamped", "    if (limit > bits_per_slot) limit = bits_per_slot;", "    ;", False,
     PINS + "test_message_status_hand_cases"),
    ("message window: unknown count completes", "(n_chunks[i] != 0 && count == limit) ? 1u : 0u;",
     "(count == limit) ? 1u : 0u;", False, PINS + "test_message_status_against_numpy"),
    ("message window: last hole instead of first", "else if (first_clear == limit) first_clear = b;",
     "else first_clear = b;", False, PINS + "test_message_status_hand_cases"),
    ("message window: recycling leaves stray bits", "      for (uint32_t b = 0; b < bits_per_slot; ++b) {",
     "      for (uint32_t b = 0; b < limit; ++b) {", False, PINS + "test_message_status_hand_cases"),
    ("message window: recycles incomplete slots", "if (recycle && complete)", "if (recycle)", False,
     PINS + "test_message_status_hand_cases"),
    ("message window: wrong slot base", "const uint64_t base = (uint64_t)i * bits_per_slot;",
     "const uint64_t base = (uint64_t)i * (bits_per_slot / 2);", False, PINS + "test_message_status_hand_cases"),
    ("ack report: cumulative run listed as a range", "if (run_start > 0) {", "if (1) {", False,
     PINS + "test_ack_report_hand_cases"),
    ("ack report: inclusive range end", "ranges[2 * runs + 1] = s; }", "ranges[2 * runs + 1] = s - 1; }", False,
     PINS + "test_ack_report_hand_cases"),
    ("multi-source 16-bit product adds", "f = op == ORC_SUM ? f + fr : f * fr;", "f = f + fr;", False,
     GATHER + "test_16bit_product_fold_runs_in_fp32_and_rounds_once"),
    ("multi-source 16-bit product rounds per source", "f = op == ORC_SUM ? f + fr : f * fr;",
     "f = op == ORC_SUM ? f + fr : f * fr; f = dtype == ORC_BF16 ? bf16_widen(orc_f32_to_bf16(f)) : orc_f16_to_f32(orc_f32_to_f16(f));",
     False, GATHER + "test_16bit_product_fold_runs_in_fp32_and_rounds_once"),
    ("multi-source 16-bit max / min copies the source",
     "t = dtype == ORC_BF16 ? orc_combine_bf16(t, r, op) : orc_combine_f16(t, r, op);", "t = r;", False,
     GATHER + "test_16bit_selection_fold_against_numpy"),
    ("multi-source 16-bit min is max",
     "t = dtype == ORC_BF16 ? orc_combine_bf16(t, r, op) : orc_combine_f16(t, r, op);",
     "t = dtype == ORC_BF16 ? orc_combine_bf16(t, r, ORC_MAX) : orc_combine_f16(t, r, ORC_MAX);", False,
     GATHER + "test_16bit_selection_fold_against_numpy"),
    ("multi-source int32 min is max",
     "t = orc_combine_i32(t, ((const int32_t*)((const char*)recv_stage + d->src_off[j]))[i], op);",
     "t = orc_combine_i32(t, ((const int32_t*)((const char*)recv_stage + d->src_off[j]))[i], op == ORC_MIN ? ORC_MAX : op);",
     False, GATHER + "test_int32_min_fold_against_numpy"),
    ("bf16 narrowing has no NaN branch",
     "if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x0040u);", ";", False,
     PINS + "test_narrowing_a_nan_gives_a_quiet_nan_of_the_same_sign"),
    ("bf16 NaN not quieted",
     "if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x0040u);",
     "if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x0001u);", False,
     PINS + "test_narrowing_a_nan_gives_a_quiet_nan_of_the_same_sign"),
    ("binary16 narrowing has no NaN branch",
     "if (mag > 0x7F800000u) return (uint16_t)(sign | 0x7E00u | ((mag >> 13) & 0x1FFu)); /* NaN, quieted */", ";", False,
     PINS + "test_narrowing_a_nan_gives_a_quiet_nan_of_the_same_sign"),
    ("segmentation: slots packed at the chunk size", "unsigned char* to = (unsigned char*)stage + stage_off + i * slot_stride;",
     "unsigned char* to = (unsigned char*)stage + stage_off + i * chunk_bytes;", False,
     SEGMENT + "test_whole_chunks_are_a_reshape"),
    ("segmentation: source offset ignored", "(const unsigned char*)tensor + tensor_off + i * chunk_bytes;",
     "(const unsigned char*)tensor + i * chunk_bytes;", False, SEGMENT + "test_ragged_tail_and_concatenation"),
    ("segmentation: last chunk padded to full length", "const uint64_t len = i + 1 < n ? chunk_bytes : last_len;",
     "const uint64_t len = chunk_bytes;", False, SEGMENT + "test_ragged_tail_and_concatenation"),
    ("segmentation: no mark at a message boundary", "const uint32_t mark = (csn == 255u || i + 1 == n) ? 1u : 0u;",
     "const uint32_t mark = (i + 1 == n) ? 1u : 0u;", False, SEGMENT + "test_headers_follow_the_field_widths"),
    ("segmentation: message id does not advance", "const uint32_t msg = (uint32_t)((msg_id + number / 256u) % 128u);",
     "const uint32_t msg = msg_id;", False, SEGMENT + "test_headers_follow_the_field_widths"),
    ("segmentation: numbering ignores the first sequence number", "const uint64_t number = (uint64_t)first_csn + i;",
     "const uint64_t number = i;", False, SEGMENT + "test_headers_follow_the_field_widths"),
    ("segmentation: record offset relative to the first slot", "descs[i].stage_off = stage_off + i * slot_stride;",
     "descs[i].stage_off = i * slot_stride;", False, SEGMENT + "test_whole_chunks_are_a_reshape"),
    ("binary16 NaN loses its sign",
     "if (mag > 0x7F800000u) return (uint16_t)(sign | 0x7E00u | ((mag >> 13) & 0x1FFu)); /* NaN, quieted */",
     "if (mag > 0x7F800000u) return (uint16_t)(0x7E00u | ((mag >> 13) & 0x1FFu));", False,
     PINS + "test_narrowing_a_nan_gives_a_quiet_nan_of_the_same_sign"),
]


def _plant_and_run(tmp, k):
    name, old, new, every, pin = MISTAKES[k]
    src = open(os.path.join(ROOT, "oracle", "chunk_oracle.c")).read()
    assert old in src, f"{name}: the oracle no longer contains the text this mistake replaces"
    mutant = src.replace(old, new) if every else src.replace(old, new, 1)
    d = os.path.join(tmp, f"m{k}")
    os.makedirs(d)
    c, lib = os.path.join(d, "chunk_oracle.c"), os.path.join(d, "libchunk_oracle.so")
    open(c, "w").write(mutant)
    subprocess.check_call(["gcc", *oracle.CFLAGS, "-pthread", f"-I{os.path.join(ROOT, 'oracle')}", c,
                           os.path.join(ROOT, "oracle", "chunk_threaded.c"), "-o", lib])
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", pin], cwd=ROOT,
                       capture_output=True, text=True, env={**os.environ, "CHUNK_ORACLE_LIB": lib})
    return name, pin, r.returncode, r.stdout[-400:]


def test_every_planted_mistake_is_caught(tmp_path):
    with concurrent.futures.ThreadPoolExecutor(max_workers=6) as pool:
        results = list(pool.map(lambda k: _plant_and_run(str(tmp_path), k), range(len(MISTAKES))))
    survived = [(n, p, out) for n, p, rc, out in results if rc != 1]   # 1 = tests ran and some failed
    assert not survived, survived


def test_the_unmodified_oracle_passes_through_the_same_route(tmp_path):
    """The route itself (build a copy, load it through CHUNK_ORACLE_LIB, run a pin) passes when
    nothing is planted, so a failure above is the mistake's doing."""
    lib = os.path.join(str(tmp_path), "libchunk_oracle.so")
    subprocess.check_call(["gcc", *oracle.CFLAGS, "-pthread", os.path.join(ROOT, "oracle", "chunk_oracle.c"),
                           os.path.join(ROOT, "oracle", "chunk_threaded.c"), "-o", lib])
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        PINS + "test_message_status_hand_cases", PINS + "test_exactly_once_all_ones"], cwd=ROOT,
                       capture_output=True, text=True, env={**os.environ, "CHUNK_ORACLE_LIB": lib})
    assert r.returncode == 0, r.stdout[-600:]
