"""Mutation check of the oracle's pins: plant one plausible mistake at a time in
a copy of the oracle's source (a dropped term, an off-by-one, a transposed
index, a wrong tie rule), build it on the CPU, and require that at least one
pin of test_oracle_pins fails.  The mistakes live only in the temporary copy.
"""
import os
import subprocess
import sys

import pytest

import oracle
from tests import test_oracle_pins as pins

SRC = os.path.join(os.path.dirname(oracle.__file__), "mcr_oracle.cpp")

# (name, text in the source, replacement)
MUTANTS = [
    ("bf16_truncates", "round_up = true;\n  } else if (discarded < half)", "round_up = false;\n  } else if (discarded < half)"),
    ("bf16_tie_always_up", "round_up = (kept & 1u) != 0u;", "round_up = true;"),
    ("bf16_tie_always_down", "round_up = (kept & 1u) != 0u;", "round_up = false;"),
    ("bf16_nan_to_inf", "return static_cast<uint16_t>((u >> 16) | 0x0040u);", "return static_cast<uint16_t>(u >> 16);"),
    ("f16_tie_rounds_up", "if (rem > 0.5 || (rem == 0.5 && std::fmod(n, 2.0) == 1.0)) n += 1.0;", "if (rem >= 0.5) n += 1.0;"),
    ("f16_truncates", "if (rem > 0.5 || (rem == 0.5 && std::fmod(n, 2.0) == 1.0)) n += 1.0;", "if (rem > 2.0) n += 1.0;"),
    ("f16_subnormal_quantum_shrinks", "  if (E < -14) E = -14;\n", ""),
    ("f16_no_carry_into_next_binade", "  if (n == 2048.0) {\n    E += 1;\n    n = 1024.0;\n  }", "  if (n == 2048.0) {\n    n = 2047.0;\n  }"),
    ("f16_widen_subnormal_scale", "std::ldexp(static_cast<float>(frac), -24)", "std::ldexp(static_cast<float>(frac), -25)"),
    ("i32_sum_saturates", "default: return static_cast<int32_t>(static_cast<uint32_t>(acc) + static_cast<uint32_t>(x));", "default: { const int64_t w = static_cast<int64_t>(acc) + x; return static_cast<int32_t>(w > 2147483647 ? 2147483647 : (w < -2147483647 - 1 ? -2147483647 - 1 : w)); }"),
    ("i32_max_unsigned", "case OP_MAX: return x > acc ? x : acc;\n    case OP_MIN: return x < acc ? x : acc;\n    case OP_PROD: return static_cast<int32_t>(static_cast<uint32_t>(acc)", "case OP_MAX: return static_cast<uint32_t>(x) > static_cast<uint32_t>(acc) ? x : acc;\n    case OP_MIN: return x < acc ? x : acc;\n    case OP_PROD: return static_cast<int32_t>(static_cast<uint32_t>(acc)"),
    ("reduce_starts_from_zero", "float acc = load_elem(bufs[0], i, dtype);\n  for (int p = 1;", "float acc = 0.0f;\n  for (int p = 0;"),
    ("reduce_drops_last_rank", "for (int p = 1; p < P; ++p) {\n    acc = combine(acc, load_elem", "for (int p = 1; p < P - 1; ++p) {\n    acc = combine(acc, load_elem"),
    ("reduce_reverse_order", "float acc = load_elem(bufs[0], i, dtype);\n  for (int p = 1; p < P; ++p) {\n    acc = combine(acc, load_elem(bufs[p], i, dtype), op);",
     "float acc = load_elem(bufs[P - 1], i, dtype);\n  for (int p = 1; p < P; ++p) {\n    acc = combine(acc, load_elem(bufs[P - 1 - p], i, dtype), op);"),
    ("avg_divides", "acc = acc * scale;", "acc = acc / static_cast<float>(P);"),
    ("allreduce_writes_rank0_only", "for (int r = 0; r < P; ++r) store_elem(bufs[r], i, dtype, y);", "store_elem(bufs[0], i, dtype, y);"),
    ("reduce_writes_everyone", "    store_elem(bufs[root], i, dtype, y);\n  }\n  return 0;\n}\n\n// ---- bcast", "    for (int r = 0; r < P; ++r) store_elem(bufs[r], i, dtype, y);\n  }\n  return 0;\n}\n\n// ---- bcast"),
    ("bcast_from_rank0", "static_cast<const char*>(bufs[root]) + i * s, s);", "static_cast<const char*>(bufs[0]) + i * s, s);"),
    ("gatherv_displ_not_advanced", "    displ += counts[p];\n  }\n  return 0;\n}\n\nint orc_scatterv", "    displ += counts[0];\n  }\n  return 0;\n}\n\nint orc_scatterv"),
    ("scatterv_ignores_displ", "static_cast<const char*>(root_in) + (displ + j) * s, s);", "static_cast<const char*>(root_in) + j * s, s);"),
    ("max_is_min", "case OP_MAX: return (x > acc || x != x) ? x : acc;", "case OP_MAX: return (x < acc || x != x) ? x : acc;"),
    ("min_drops_nan", "case OP_MIN: return (x < acc || x != x) ? x : acc;", "case OP_MIN: return (x < acc) ? x : acc;"),
    ("prod_adds", "case OP_PROD: return acc * x;", "case OP_PROD: return acc + x;"),
    ("displs_alltoallv_tables_swapped", "const int64_t from = sdispls[p * P + r];\n      const int64_t to = rdispls[r * P + p];", "const int64_t from = rdispls[r * P + p];\n      const int64_t to = sdispls[p * P + r];"),
    ("displs_rdispls_indexed_by_sender", "const int64_t to = rdispls[r * P + p];", "const int64_t to = rdispls[p * P + r];"),
    ("displs_gatherv_ignored", "static_cast<char*>(root_out) + (displs[p] + j) * s, static_cast<const char*>(in[p]) + j * s, s);", "static_cast<char*>(root_out) + (displs[0] + j) * s, static_cast<const char*>(in[p]) + j * s, s);"),
    ("displs_scatterv_on_the_wrong_side", "std::memcpy(static_cast<char*>(out[r]) + j * s, static_cast<const char*>(root_in) + (displs[r] + j) * s, s);", "std::memcpy(static_cast<char*>(out[r]) + (displs[r] + j) * 0 + j * s, static_cast<const char*>(root_in) + j * s, s);"),
    ("rs_wrong_slice", "reduce_at(in, static_cast<size_t>(r) * b + j, dtype, op, P);", "reduce_at(in, j, dtype, op, P);"),
    ("allgather_transposed", "static_cast<char*>(out[r]) + (static_cast<size_t>(p) * m + j) * s,\n                    static_cast<const char*>(in[p]) + j * s, s);",
     "static_cast<char*>(out[r]) + (static_cast<size_t>(r) * m + j) * s,\n                    static_cast<const char*>(in[p]) + j * s, s);"),
    ("alltoall_no_transpose", "static_cast<const char*>(in[p]) + (static_cast<size_t>(r) * b + k) * s, s);",
     "static_cast<const char*>(in[p]) + (static_cast<size_t>(p) * b + k) * s, s);"),
    ("alltoallv_sdispl_inclusive", "for (int q = 0; q < r; ++q) sdispl += S[p * P + q];", "for (int q = 0; q <= r; ++q) sdispl += S[p * P + q];"),
    ("alltoallv_S_transposed", "const int64_t cnt = S[p * P + r];", "const int64_t cnt = S[r * P + p];"),
    ("alltoallv_back_counts_not_transposed", "const int64_t back = S[b * P + a];", "const int64_t back = S[a * P + b];"),
    ("alltoallv_back_sdispl_along_the_row", "for (int q = 0; q < b; ++q) sdispl += S[q * P + a];", "for (int q = 0; q < b; ++q) sdispl += S[a * P + q];"),
    ("alltoallv_back_sdispl_inclusive", "for (int q = 0; q < b; ++q) sdispl += S[q * P + a];", "for (int q = 0; q <= b; ++q) sdispl += S[q * P + a];"),
    ("route_capacity_off_by_one", "pos[static_cast<size_t>(t)] >= C) {", "pos[static_cast<size_t>(t)] > C) {"),
    ("route_base_inclusive", "base[static_cast<size_t>(e)] = run;\n    run += c;", "run += c;\n    base[static_cast<size_t>(e)] = run;"),
    ("route_counts_unclamped", "const int64_t c = seen[static_cast<size_t>(e)] < C ? seen[static_cast<size_t>(e)] : C;", "const int64_t c = seen[static_cast<size_t>(e)];"),
    ("route_rank_map_strided", "for (int e = r * per_rank; e < (r + 1) * per_rank; ++e) s += counts[e];", "for (int e = r; e < E; e += P) s += counts[e];"),
    ("layout_first_not_reset_per_rank", "for (int e2 = (e / per_rank) * per_rank; e2 < e; ++e2) first += expert_rows[e2];", "for (int e2 = 0; e2 < e; ++e2) first += expert_rows[e2];"),
    ("layout_sources_not_stacked", "      block_first[p * E + e] = first + above;\n      above += counts[p * E + e];", "      block_first[p * E + e] = first + above;"),
    ("by_expert_wrong_rank", "      std::memcpy(static_cast<char*>(recv[e / per_rank]) + static_cast<size_t>(row) * rb,", "      std::memcpy(static_cast<char*>(recv[e % P]) + static_cast<size_t>(row) * rb,"),
    ("topk_second_choice_reads_first_token", "static_cast<const char*>(tok[p]) + static_cast<size_t>(t) * rb, rb);\n      }\n    }", "static_cast<const char*>(tok[p]) + static_cast<size_t>(a % (K * T)) * 0 + static_cast<size_t>(k == 0 ? t : 0) * rb, rb);\n      }\n    }"),
    ("topk_sum_reversed", "for (int k = 0; k < K; ++k) {\n          const size_t a = static_cast<size_t>(k) * T + t;\n          if (!src[a]) continue;", "for (int k = K - 1; k >= 0; --k) {\n          const size_t a = static_cast<size_t>(k) * T + t;\n          if (!src[a]) continue;"),
    ("topk_gate_of_first_choice", "const float g = gate ? gate[p][a] : 1.0f;", "const float g = gate ? gate[p][t] : 1.0f;"),
    ("topk_sum_starts_from_zero", "acc = first ? term : acc + term;", "acc = acc + term;"),
    ("unpack_dropped_not_zeroed", "std::memset(dst, 0, rb);\n      continue;", "continue;"),
    ("unpack_gate_of_slot", "const float g = gate[t];", "const float g = gate[slot[t]];"),
    ("pack_gathers_instead", "std::memcpy(static_cast<char*>(out) + static_cast<size_t>(slot[t]) * rb,\n                static_cast<const char*>(in) + static_cast<size_t>(t) * rb, rb);",
     "std::memcpy(static_cast<char*>(out) + static_cast<size_t>(t) * rb,\n                static_cast<const char*>(in) + static_cast<size_t>(slot[t]) * rb, rb);"),
    ("dlrm_owner_blocked", "const int owner = t % P;\n        const int local = t / P;\n        const size_t src_row = static_cast<size_t>(local) * static_cast<size_t>(batch) +\n                               static_cast<size_t>(r) * static_cast<size_t>(bl) + static_cast<size_t>(b);\n        const size_t dst_row = static_cast<size_t>(b) * static_cast<size_t>(n_tables) + static_cast<size_t>(t);\n        std::memcpy(static_cast<char*>(out[r])",
     "const int owner = t % P;\n        const int local = t / P;\n        const size_t src_row = static_cast<size_t>(local) * static_cast<size_t>(batch) +\n                               static_cast<size_t>(r) * static_cast<size_t>(bl) + static_cast<size_t>(b);\n        const size_t dst_row = static_cast<size_t>(t) * static_cast<size_t>(bl) + static_cast<size_t>(b);\n        std::memcpy(static_cast<char*>(out[r])"),
    ("plan_closes_when_full_exactly", "cur_fill + n > B)) {", "cur_fill + n >= B)) {"),
    ("plan_oversize_shares_bucket", "if (open && (n > B || cur_fill + n > B)) {", "if (open && (cur_fill + n > B && n <= B)) {"),
    ("fuse_ignores_offset", "std::memcpy(static_cast<char*>(flat) + (offset[i] + j) * s,", "std::memcpy(static_cast<char*>(flat) + j * s,"),
    ("lookup_ceiling_rule", "if (sizes[i] <= bytes) pick = i;", "if (sizes[i] < bytes) pick = (i + 1 < n_rows) ? i + 1 : i;"),
]


@pytest.fixture
def source():
    with open(SRC) as f:
        return f.read()


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_mutant_is_caught(name, old, new, source, tmp_path):
    assert source.count(old) >= 1, f"mutation site for {name} no longer in the oracle source"
    mutated = source.replace(old, new, 1)
    cpp = tmp_path / "mutant.cpp"
    so = tmp_path / "mutant.so"
    cpp.write_text(mutated)
    subprocess.check_call(["g++", *[f for f in oracle.CXXFLAGS if not f.startswith("-W")], "-w", "-o", str(so), str(cpp)])
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    proc = subprocess.run([sys.executable, "-m", "tests.mutant_runner", str(so)], cwd=root,
                          stdout=subprocess.PIPE, stderr=subprocess.DEVNULL, text=True, timeout=300)
    # 3 = a pin failed; a negative code = the planted mistake corrupted memory and the child died
    assert proc.returncode != 0, f"no pin notices the planted mistake '{name}'"
    assert proc.returncode == 3 or proc.returncode < 0, (name, proc.returncode, proc.stdout)
