"""Are the oracle's pins sharp?  One mistake at a time is planted in a COPY of the oracle's sources (a dropped
term, a wrong sign, a wrong or transposed index, an off-by-one in a rule), the copy is built into a library of
its own in a temporary directory, and the pin tests of the touched file are run against it in a child process:
they must fail.  Nothing here touches the GPU path or the oracle that the other tests use."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor
from pathlib import Path

import pytest

import oracle

ROOT = Path(__file__).resolve().parents[1]
PINS = {"spmv_oracle.cpp": "tests/test_oracle_spmv.py", "analysis_oracle.cpp": "tests/test_oracle_analysis.py",
        "spmm_oracle.cpp": "tests/test_oracle_spmm.py", "formats_oracle.cpp": "tests/test_oracle_formats.py"}

# (file, text as it stands, text with the mistake, what the mistake is)
MUTANTS = [
    ("spmv_oracle.cpp", "acc += p;", "acc -= p;", "products subtracted"),
    ("spmv_oracle.cpp", "if (beta != 0.0f) r += static_cast<double>(beta) * static_cast<double>(y0[i]);", ";", "beta*y0 dropped"),
    ("spmv_oracle.cpp", "if (beta != 0.0f) r += static_cast<double>(beta)", "if (beta != 0.0f) r -= static_cast<double>(beta)", "beta*y0 subtracted"),
    ("spmv_oracle.cpp", "static_cast<double>(x[j])", "static_cast<double>(x[i < n ? i : j])", "x taken at the row index (f32)"),
    ("spmv_oracle.cpp", "bf16_bits_to_float(x[j])", "bf16_bits_to_float(x[i < n ? i : j])", "x taken at the row index (bf16)"),
    ("spmv_oracle.cpp", "S += std::fabs(p);", "S += p;", "S without the absolute value"),
    ("spmv_oracle.cpp", "for (int64_t k = rowptr[i]; k < rowptr[i + 1]; ++k)", "for (int64_t k = rowptr[i] + 1; k < rowptr[i + 1]; ++k)", "first entry of every row dropped"),
    ("spmv_oracle.cpp", "for (int64_t k = rowptr[i]; k < rowptr[i + 1]; ++k)", "for (int64_t k = rowptr[i]; k + 1 < rowptr[i + 1]; ++k)", "last entry of every row dropped"),
    ("spmv_oracle.cpp", "static_cast<uint32_t>(b) << 16", "static_cast<uint32_t>(b) << 15", "bf16 widened by the wrong shift"),
    ("spmv_oracle.cpp", "double r = static_cast<double>(alpha) * acc;", "double r = acc;", "alpha dropped"),
    ("spmv_oracle.cpp", "const double p = static_cast<double>(vals[k]) * static_cast<double>(x[j]);", "const double p = vals[k] * x[j];", "product rounded to float"),
    ("spmv_oracle.cpp", "const int32_t j = colidx[k];", "const int32_t j = colidx[k == rowptr[i] ? k : k - 1];", "column index taken one entry early"),
    ("analysis_oracle.cpp", "while (cap < len) {", "while (cap <= len) {", "bins off by one at powers of two"),
    ("analysis_oracle.cpp", "if (len == 0) ++empty;", "if (len <= 1) ++empty;", "rows of one entry counted as empty"),
    ("analysis_oracle.cpp", "if (held + len > block_nnz) break;", "if (held + len >= block_nnz) break;", "row blocks close one entry early"),
    ("analysis_oracle.cpp", "if (r - first >= rows_max) break;", "if (r - first > rows_max) break;", "row blocks take one row too many"),
    ("analysis_oracle.cpp", "if (r == first) ++r;  // a single row that is longer than block_nnz", "if (r == first) r += 2;", "an over-long row swallows its successor"),
    ("analysis_oracle.cpp", "rowptr[i + 1] > j)", "rowptr[i + 1] >= j)", "merge path moves down instead of right on a tie"),
    ("analysis_oracle.cpp", "if (step == p * ipc || step == T) {", "if (step == p * ipc + 1 || step == T) {", "merge path diagonals shifted by one"),
    ("analysis_oracle.cpp", "rank * vec_elems + colidx[k] % vec_elems", "rank + colidx[k] % vec_elems", "window position not scaled by the vector length"),
    ("analysis_oracle.cpp", "xv_start[total + static_cast<int64_t>(j)] = keys[j] * vec_elems;", "xv_start[total + static_cast<int64_t>(j)] = keys[j];", "x vector start not scaled"),
    ("analysis_oracle.cpp", "keys.erase(std::unique(keys.begin(), keys.end()), keys.end());", ";", "duplicate x vectors kept"),
    ("analysis_oracle.cpp", "return 4 * nb * V <= nnz ? 1 : 0;", "return nb * V <= nnz ? 1 : 0;", "window rule without its factor 4"),
    ("analysis_oracle.cpp", "if (V > max_vectors) return 0;", "if (V >= max_vectors) return 0;", "window rule refuses the largest allowed window"),
    ("analysis_oracle.cpp", "cb_col[k] = static_cast<int32_t>(colidx[e] - b * width);", "cb_col[k] = static_cast<int32_t>(colidx[e]);", "column not made relative to its block"),
    ("analysis_oracle.cpp", "cb_src[k] = static_cast<int32_t>(e);", "cb_src[k] = static_cast<int32_t>(e + 1);", "source position off by one"),
    ("analysis_oracle.cpp", "if (colidx[e] / width == b) {", "if (colidx[e] / width == C - 1 - b) {", "column blocks in reverse order"),
    ("analysis_oracle.cpp", "while (G < 64 && 16 * G < mean) G *= 2;", "while (G < 64 && 8 * G < mean) G *= 2;", "tile shape from the wrong lane rule"),
    ("analysis_oracle.cpp", "if (max_len > block_nnz) return 5;", "if (max_len >= block_nnz) return 5;", "plan rule off by one"),
    ("analysis_oracle.cpp", "while (G < 64 && 8 * static_cast<int64_t>(G) < mean_up) G *= 2;", "while (G < 64 && 8 * static_cast<int64_t>(G) <= mean_up) G *= 2;", "vector lanes off by one"),
    ("analysis_oracle.cpp", "n > 2 * width && C <= 16", "n >= 2 * width && C <= 16", "column block rule off by one"),
    ("analysis_oracle.cpp", "if (rowptr[row_blocks[b]] % 8 != 0) return 0;", ";", "grouped positions: block starts not checked"),
    ("analysis_oracle.cpp", "for (int64_t i = 1; i < 8; ++i)\n            if (lidx[8 * g + i] != lidx[8 * g] + i) return 0;", "for (int64_t i = 1; i < 7; ++i)\n            if (lidx[8 * g + i] != lidx[8 * g] + i) return 0;", "grouped positions: last of a group not checked"),
    ("analysis_oracle.cpp", "for (int64_t g = 0; g < nnz / 8; ++g)\n        for (int64_t i = 1; i < 8; ++i)", "for (int64_t g = 0; g < (nnz + 7) / 8; ++g)\n        for (int64_t i = 1; i < 8; ++i)", "grouped positions: the tail taken for a group"),
    ("analysis_oracle.cpp", "if (nnz < 8) return 0;\n    for (int64_t b = 0; b < nb; ++b)\n        if (rowptr[row_blocks[b]] % 8", "if (nnz < 0) return 0;\n    for (int64_t b = 0; b < nb; ++b)\n        if (rowptr[row_blocks[b]] % 8", "grouped positions: fewer than eight entries accepted"),
    ("analysis_oracle.cpp", "if (vectors < 0 || 4 * vectors < 3 * entries) return 0;  // clustered", "if (vectors < 0 || 4 * vectors <= 3 * entries) return 0;  // clustered", "column block rule: scatter threshold off by one"),
    ("analysis_oracle.cpp", "if (vectors < 0 || 4 * vectors < 3 * entries) return 0;  // clustered", "if (4 * vectors < 3 * entries) return 0;  // clustered", "column block rule: uncounted windows taken for scattered"),
    ("analysis_oracle.cpp", "if (vectors < 0 || 4 * vec_elems * vectors < 3 * entries) return 0;", "if (vectors < 0 || 4 * vectors < 3 * entries) return 0;", "two-pass on groups: scatter measured per entry"),
    ("analysis_oracle.cpp", "n * elem_bytes >= (int64_t{1} << 20) && ng >= 3", "n * elem_bytes > (int64_t{1} << 20) && ng >= 3", "two-pass on groups: x threshold off by one"),
    ("analysis_oracle.cpp", "C * P <= (int64_t{1} << 24) &&\n            8 * C * P <= ng)", "C * P <= (int64_t{1} << 24) &&\n            8 * C * P <= nnz)", "two-pass on groups: tiles measured in entries"),
    ("analysis_oracle.cpp", "if (!(plan == 4 || plan == 5) || !group_aligned) return 0;", "if (!group_aligned) return 0;", "two-pass on groups: taken from any plan"),
    ("analysis_oracle.cpp", "int64_t k = total >= static_cast<int64_t>(waves) * resident * floor ? waves : 1;", "int64_t k = waves;", "piece size: small matrices cut for several rounds too"),
    ("analysis_oracle.cpp", "if (pieces <= k * resident) return static_cast<int32_t>(t < floor ? floor : t);", "if (pieces <= k * resident) return static_cast<int32_t>(t);", "piece size: no floor"),
    ("analysis_oracle.cpp", "for (int64_t c = 0; c < C; ++c) pieces += (groups[c] + t - 1) / t;", "for (int64_t c = 0; c < C; ++c) pieces += groups[c] / t;", "piece size: a block's last, shorter piece not counted"),
    ("analysis_oracle.cpp", "if (i < m && rowptr[i] < j && j <= rowptr[i + 1] && rowptr[i + 1] - rowptr[i] <= snap) j = rowptr[i];", "if (i < m && rowptr[i] < j && j < rowptr[i + 1] && rowptr[i + 1] - rowptr[i] <= snap) j = rowptr[i];", "two-pass chunks: a row whose entries are all taken but which is not finished is left cut"),
    ("analysis_oracle.cpp", "if (i < m && rowptr[i] < j && j <= rowptr[i + 1] && rowptr[i + 1] - rowptr[i] <= snap) j = rowptr[i];", "if (i < m && rowptr[i] < j && j <= rowptr[i + 1] && rowptr[i + 1] - rowptr[i] < snap) j = rowptr[i];", "two-pass chunks: rows of exactly snap entries cut"),
    ("analysis_oracle.cpp", "if (i < m && rowptr[i] < j && j <= rowptr[i + 1] && rowptr[i + 1] - rowptr[i] <= snap) j = rowptr[i];", "if (i < m && rowptr[i] < j && j <= rowptr[i + 1] && rowptr[i + 1] - rowptr[i] <= snap) j = rowptr[i + 1];", "two-pass chunks: the cut moved forward instead of back"),
    ("analysis_oracle.cpp", "const int64_t P = oracle_merge_path_snapped(m, nnz, rowptr, items, snap, tp_row, tp_nz);", "const int64_t P = oracle_merge_path_snapped(m, nnz, rowptr, items, 0, tp_row, tp_nz);", "two-pass layout: chunks not snapped"),
    ("analysis_oracle.cpp", "col[s1] = static_cast<uint16_t>(colidx[k] - (c << shift));", "col[s1] = static_cast<uint16_t>(colidx[k]);", "two-pass: column not made relative to its block"),
    ("analysis_oracle.cpp", "pos[s2] = static_cast<uint16_t>(k - tp_nz[pp]);", "pos[s2] = static_cast<uint16_t>(k - tp_nz[pp] + 1);", "two-pass: position in the chunk off by one"),
    ("analysis_oracle.cpp", "if (o % 4 == 0) from[s2 / 4] = static_cast<int32_t>(s1 / 4);", "if (o % 4 == 0) from[s2 / 4] = static_cast<int32_t>(s2 / 4);", "two-pass: products fetched as if they lay in the reduce order"),
    ("analysis_oracle.cpp", "if (o % 4 == 0) from[s2 / 4] = static_cast<int32_t>(s1 / 4);", "if (o % 4 == 0) from[s1 / 4] = static_cast<int32_t>(s2 / 4);", "two-pass: the map of groups taken the other way round"),
    ("analysis_oracle.cpp", "start2[static_cast<size_t>(c * P + pp)] = slot;\n            slot += (cnt[static_cast<size_t>(c * P + pp)] + 3) / 4 * 4;", "start2[static_cast<size_t>(c * P + pp)] = slot;\n            slot += cnt[static_cast<size_t>(c * P + pp)];", "two-pass: reduce order not padded"),
    ("analysis_oracle.cpp", "while (tp_nz[p + 1] <= k) ++p;", "while (tp_nz[p + 1] < k) ++p;", "two-pass: an entry on a split goes to the chunk before"),
    ("analysis_oracle.cpp", "block_first_group + i * ((groups + pieces - 1) / pieces)", "block_first_group + i * piece_groups", "two-pass: pieces filled to the cap instead of cut evenly"),
    ("analysis_oracle.cpp", "const int64_t pieces = (groups + piece_groups - 1) / piece_groups;\n        for (int64_t i = 0; i < pieces; ++i) {", "const int64_t pieces = groups / piece_groups + 1;\n        for (int64_t i = 0; i < pieces; ++i) {", "two-pass: one piece too many when the cap divides the block"),
    ("analysis_oracle.cpp", "8 * C * P <= nnz)", "8 * C * P < nnz)", "two-pass rule off by one"),
    ("analysis_oracle.cpp", "C * P <= (int64_t{1} << 24) &&", "C * P < (int64_t{1} << 24) &&", "two-pass rule: tile limit off by one"),
    ("analysis_oracle.cpp", "if (vectors < 0 || 4 * vectors < 3 * entries) return 0;\n    return ((plan == 4 || plan == 5) && 16 * n", "if (vectors < 0 || 4 * vectors <= 3 * entries) return 0;\n    return ((plan == 4 || plan == 5) && 16 * n", "two-pass rule: scatter threshold off by one"),
    ("analysis_oracle.cpp", "if (vectors < 0 || 4 * vectors < 3 * entries) return 0;\n    return ((plan == 4 || plan == 5) && 16 * n", "if (4 * vectors < 3 * entries) return 0;\n    return ((plan == 4 || plan == 5) && 16 * n", "two-pass rule: uncounted windows taken for scattered"),
    ("analysis_oracle.cpp", "if (in_block <= block_nnz) *entries += in_block;", "*entries += in_block;", "scatter counts: over-long rows counted"),
    ("analysis_oracle.cpp", "if (in_block <= block_nnz) *entries += in_block;", "if (in_block < block_nnz) *entries += in_block;", "scatter counts: full blocks left out"),
    ("analysis_oracle.cpp", "nnz >= 3 * (int64_t{1} << 21) && C <= 65535", "nnz > 3 * (int64_t{1} << 21) && C <= 65535", "two-pass rule: entry threshold off by one"),
    ("analysis_oracle.cpp", "(plan == 4 || plan == 5) && 16 * n >= width && nnz >= 3", "(plan == 4 || plan == 5) && 16 * n > width && nnz >= 3", "two-pass rule: width threshold off by one"),
    ("analysis_oracle.cpp", "(plan == 4 || plan == 5) && 16 * n >= width && nnz >= 3", "(plan == 4 || plan == 5) && 2 * n >= width && nnz >= 3", "two-pass rule: x of 2 MiB asked for"),
    ("analysis_oracle.cpp", "if (rows_so_far == 1) {\n                    joins = true;", "if (rows_so_far >= 1) {\n                    joins = true;", "row patterns: every step accepted as the run's stride"),
    ("analysis_oracle.cpp", "} else if (step == stride.back()) {", "} else if (step >= stride.back()) {", "row patterns: a larger step joins the run"),
    ("analysis_oracle.cpp", "if (!start.empty() && rel[i] == rel[i - 1]) {", "if (!start.empty() && rel[i].size() == rel[i - 1].size()) {", "row patterns: only the lengths compared"),
    ("analysis_oracle.cpp", "if (d < 0) ok = false;", ";", "row patterns: negative offsets accepted"),
    ("analysis_oracle.cpp", "if (len > max_len) ok = false;", "if (len >= max_len) ok = false;", "row patterns: the longest allowed row refused"),
    ("analysis_oracle.cpp", "if (static_cast<int64_t>(start.size()) > max_runs) continue;", "if (static_cast<int64_t>(start.size()) >= max_runs) continue;", "row patterns: the most allowed runs refused"),
    ("analysis_oracle.cpp", "bool ok = entries <= block_nnz;", "bool ok = entries < block_nnz;", "row patterns: a full block left out"),
    ("analysis_oracle.cpp", "run_base[q] = static_cast<int32_t>(base[start[r]]);", "run_base[q] = static_cast<int32_t>(base[end - 1]);", "row patterns: base of the run's last row"),
    ("analysis_oracle.cpp", "base.push_back(len > 0 ? lidx[k] : 0);", "base.push_back(len > 0 ? lidx[k + len - 1] : 0);", "row patterns: base from the row's last entry"),
    ("analysis_oracle.cpp", "return (nnz > 0 && 2 * covered >= nnz) ? 1 : 0;", "return (nnz > 0 && 2 * covered > nnz) ? 1 : 0;", "pattern rule off by one"),
    ("spmm_oracle.cpp", "static_cast<double>(B[j * ldb + k]);", "static_cast<double>(B[j * ldb + (K - 1 - k)]);", "columns of B reversed"),
    ("spmm_oracle.cpp", "static_cast<double>(B[j * ldb + k]);", "static_cast<double>(B[j * K + k]);", "leading dimension of B ignored"),
    ("spmm_oracle.cpp", "if (beta != 0.0f) r += static_cast<double>(beta)", "if (beta != 0.0f) r -= static_cast<double>(beta)", "beta*C subtracted"),
    ("spmm_oracle.cpp", "S += std::fabs(p);", "S += p;", "S without the absolute value"),
    ("spmm_oracle.cpp", "const uint32_t u = static_cast<uint32_t>(b) << 16;\n    float f;\n    static_assert", "const uint32_t u = static_cast<uint32_t>(b) << 15;\n    float f;\n    static_assert", "bf16 widened by the wrong shift (SpMM)"),
    ("spmm_oracle.cpp", "const double p = bf16_to_double(vals[e]) * bf16_to_double(B[j * ldb + k]);", "const double p = bf16_to_double(vals[e]) * bf16_to_double(B[j * K + k]);", "leading dimension of a bf16 B ignored"),
    ("spmm_oracle.cpp", "const double p = bf16_to_double(vals[e]) * bf16_to_double(B[j * ldb + k]);", "const double p = static_cast<double>(static_cast<float>(bf16_to_double(vals[e]) * bf16_to_double(B[j * ldb + k])) * 1.0000001f);", "bf16 products rounded and scaled"),
    ("spmm_oracle.cpp", "return std::min<int64_t>((len + 3) / 4, 64);", "return std::min<int64_t>((len + 3) / 4, 63);", "row order: cap one too low"),
    ("spmm_oracle.cpp", "return std::min<int64_t>((len + 3) / 4, 64);", "return std::min<int64_t>(len / 4, 64);", "row order: key rounded down"),
    ("spmm_oracle.cpp", "return key(a) > key(b);", "return key(a) < key(b);", "row order ascending"),
    ("spmm_oracle.cpp", "t = 16 * b + 4 * q + e;", "t = 16 * b + 4 * e + q;", "packed copy: slots of a lane interleaved"),
    ("spmm_oracle.cpp", "desc[2 * g + 1] = static_cast<int32_t>((L + 3) / 4);", "desc[2 * g + 1] = static_cast<int32_t>((L + 4) / 4);", "packed copy: one step too many"),
    ("spmm_oracle.cpp", "blocks += (L + 15) / 16;", "blocks += (L + 16) / 16;", "packed copy: one block too many for rows of 16"),
    ("spmm_oracle.cpp", "256 * blocks <= 2 * nnz", "256 * blocks <= nnz", "packed copy: size rule without its factor 2"),
    ("formats_oracle.cpp", "const double p = widen_at(vals, e, dtype) * widen_at(x, col[e], dtype);", "const double p = widen_at(vals, e, dtype) * widen_at(x, row[e] < n ? row[e] : col[e], dtype);", "COO: x taken at the row index"),
    ("formats_oracle.cpp", "const double p = widen_at(vals, e, dtype) * widen_at(x, j, dtype);", "const double p = widen_at(vals, e, dtype) * widen_at(x, row[e] < n ? row[e] : j, dtype);", "CSC: x taken at the row index"),
    ("formats_oracle.cpp", "if (j == -1) continue;", "if (j == -1) return 1;", "ELL: padding refused"),
    ("formats_oracle.cpp", "const int32_t j = col_ids[i * width + s];", "const int32_t j = col_ids[s * m + i];", "ELL: read as column-major"),
    ("formats_oracle.cpp", "double r = static_cast<double>(alpha) * acc[i];", "double r = acc[i];", "alpha dropped"),
    ("formats_oracle.cpp", "y_ref[row[e]] += p;\n        S_ref[row[e]] += std::fabs(p);\n    }\n    finish", "y_ref[row[e]] = p;\n        S_ref[row[e]] += std::fabs(p);\n    }\n    finish", "COO: repeated coordinates overwrite"),
    ("analysis_oracle.cpp", "if (r < m) width = std::max<int64_t>(width, rowptr[r + 1] - rowptr[r]);", "if (r < m) width = std::max<int64_t>(width, rowptr[r + 1] - rowptr[r] - 1);", "sliced ELL: slices one entry too narrow"),
    ("analysis_oracle.cpp", "const int64_t slot = slice_ptr[s] + j * height + i;", "const int64_t slot = slice_ptr[s] + i * ((slice_ptr[s + 1] - slice_ptr[s]) / height) + j;", "sliced ELL: slices stored row by row"),
    ("analysis_oracle.cpp", "sell_col[slot] = -1;\n                sell_src[slot] = -1;", "sell_col[slot] = 0;\n                sell_src[slot] = -1;", "sliced ELL: padding marked with column 0"),
    ("analysis_oracle.cpp", "for (int64_t i = 0; i < height; ++i) {\n            const int64_t r = s * height + i;\n            if (r < m) width", "for (int64_t i = 0; i + 1 < height || i == 0; ++i) {\n            const int64_t r = s * height + i;\n            if (r < m) width", "sliced ELL: a slice's last row not measured"),
    ("analysis_oracle.cpp", "sell_src[slot] = static_cast<int32_t>(rowptr[r] + j);", "sell_src[slot] = static_cast<int32_t>(rowptr[r] + j + 1);", "sliced ELL: source position off by one"),
    ("analysis_oracle.cpp", "sell_col[slot] = colidx[rowptr[r] + j];", "sell_col[slot] = colidx[rowptr[r]];", "sliced ELL: every slot of a row holds its first column"),
    ("spmm_oracle.cpp", "keyed[static_cast<size_t>(t)] = {4 * seen[c % 4]++ + ((c - p) % 4 + 4) % 4, t};", "keyed[static_cast<size_t>(t)] = {4 * seen[c % 4]++ + c % 4, t};", "packed copy: entry order not turned by the row's position"),
    ("spmm_oracle.cpp", "keyed[static_cast<size_t>(t)] = {4 * seen[c % 4]++ + ((c - p) % 4 + 4) % 4, t};", "keyed[static_cast<size_t>(t)] = {seen[c % 4]++ + 4 * (((c - p) % 4 + 4) % 4), t};", "packed copy: entries grouped by residue instead of dealt out in turn"),
    ("spmm_oracle.cpp", "pcol[slot] = colidx[first + order[static_cast<size_t>(t)]];", "pcol[slot] = colidx[first + t];", "packed copy: columns left in storage order"),
    ("analysis_oracle.cpp", "if (c % width != 0) return 0;", ";", "group-aligned: a group may start anywhere"),
    ("analysis_oracle.cpp", "for (int64_t i = 1; i < width; ++i)\n            if (colidx[width * g + i] != c + i) return 0;", "for (int64_t i = 1; i + 1 < width; ++i)\n            if (colidx[width * g + i] != c + i) return 0;", "group-aligned: last column of a group not checked"),
    ("analysis_oracle.cpp", "if (rowptr[i] % width != 0) return 0;", ";", "group-aligned: rows may start inside a group"),
]


def build(tmp, tag, mutated_file=None, old=None, new=None):
    srcs = []
    for src in oracle.SOURCES:
        text = src.read_text()
        if src.name == mutated_file:
            assert text.count(old) >= 1, (mutated_file, old)
            text = text.replace(old, new)
        dst = tmp / f"{tag}_{src.name}"
        dst.write_text(text)
        srcs.append(str(dst))
    lib = tmp / f"lib_{tag}.so"
    subprocess.run(["g++", "-O1", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off", "-o", str(lib)] + srcs, check=True)
    return lib


def pins_pass(lib, module):
    env = dict(os.environ, SPMV_ORACLE_LIB=str(lib))
    r = subprocess.run([sys.executable, "-m", "pytest", module, "-x", "-q", "-p", "no:cacheprovider"], cwd=ROOT, env=env,
                       stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    return r.returncode == 0, r.stdout[-600:]


def test_every_planted_mistake_is_caught(tmp_path):
    with ThreadPoolExecutor(max_workers=6) as pool:
        control = build(tmp_path, "control")
        clean = list(pool.map(lambda mod: pins_pass(control, mod), PINS.values()))
        assert all(ok for ok, _ in clean), [tail for ok, tail in clean if not ok]    # the same build, unchanged, passes
        libs = list(pool.map(lambda kv: build(tmp_path, f"m{kv[0]}", kv[1][0], kv[1][1], kv[1][2]), enumerate(MUTANTS)))
        results = list(pool.map(lambda kv: pins_pass(kv[0], PINS[kv[1][0]]), zip(libs, MUTANTS)))
    survivors = [(m[0], m[3]) for m, (ok, _) in zip(MUTANTS, results) if ok]
    assert not survivors, f"pins that let a planted mistake through: {survivors}"
