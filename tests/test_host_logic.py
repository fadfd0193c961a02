"""CPU-only checks of the product's host logic: the C ABI loads and exports what the header
declares, arguments are validated before any GPU call, the launch planner covers every row,
and the fp32 ExtExp arithmetic (compiled for the host from the kernel's own header) meets the
accuracy the paper states."""
import ctypes
import math
import os
import re
import subprocess
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "softmax_tp.h")


@pytest.fixture(scope="module")
def B():
    from paper_2001_04438_amd import binding, buildlib
    if not os.path.exists(binding.LIB_PATH):
        buildlib.build()
    binding.lib()
    yield binding
    binding.softmax_tp_tune_reset()


def declared_symbols():
    text = open(HEADER).read()
    return re.findall(r"^TP_API\s+(?:const\s+)?\w+\s*\*?\s*(\w+)\s*\(", text, flags=re.M)


def test_library_exports_every_declared_symbol(B):
    names = declared_symbols()
    assert len(names) >= 14 and "softmax2p_f32" in names and "softmax2p_bf16io" in names
    raw = ctypes.CDLL(B.LIB_PATH)
    for name in names:
        assert hasattr(raw, name), name
    assert set(names) == set(B.ENTRY_POINTS)


def test_arguments_are_validated_before_any_gpu_call(B):
    L = B.lib()
    for fn in (L.softmax2p_f32, L.softmax3p_recompute_f32, L.softmax3p_reload_f32, L.softmax2p_bf16io):
        assert fn(None, None, 0, 0, None) == 0
        assert fn(None, None, 0, 10, None) == 0
        assert fn(None, None, 10, 0, None) == 0
        assert fn(None, None, -1, 4, None) == B.TP_ERR_NEGATIVE
        assert fn(None, None, 4, -1, None) == B.TP_ERR_NEGATIVE
        assert fn(None, 64, 1, 4, None) == B.TP_ERR_NULL
        assert fn(64, None, 1, 4, None) == B.TP_ERR_NULL
        assert fn(64, 64, 1 << 40, 1 << 40, None) == B.TP_ERR_TOO_LARGE
        assert fn(65, 64, 1, 4, None) == B.TP_ERR_ALIGN
    assert L.softmax2p_f32(66, 64, 1, 4, None) == B.TP_ERR_ALIGN      # fp32 needs 4-byte alignment
    assert L.softmax_tp_extexp_f32(None, None, None, -3, None) == B.TP_ERR_NEGATIVE
    assert L.softmax_tp_extexp_f32(None, 64, 64, 3, None) == B.TP_ERR_NULL
    assert L.softmax2p_f32_pass1(64, None, 1, 4, None) == B.TP_ERR_NULL
    assert L.softmax2p_f32_pass2(64, None, 64, 1, 4, None) == B.TP_ERR_NULL
    assert L.softmax2p_f32_pass2(64, 68, 64, 1, 4, None) == B.TP_ERR_ALIGN  # pairs need 8 bytes
    assert L.softmax_tp_stream_copy_f32(None, 64, 5, None) == B.TP_ERR_NULL
    # the entry point on static scratch: usual checks first, then the size of its partial results
    assert L.softmax2p_f32_static(None, 64, 1, 4, None) == B.TP_ERR_NULL
    assert L.softmax2p_f32_static(64, 64, -1, 4, None) == B.TP_ERR_NEGATIVE
    assert L.softmax2p_f32_static(None, None, 0, 7, None) == 0
    assert B.softmax_tp_plan(200_000, 100_000).path == 2
    assert L.softmax2p_f32_static(64, 64, 200_000, 100_000, None) == B.TP_ERR_SCRATCH
    assert "scratch" in B.strerror(B.TP_ERR_SCRATCH)
    assert L.softmax_tp_plan(1, 1, 3, 1, ctypes.byref(B.Plan())) == B.TP_ERR_TUNING
    assert L.softmax_tp_plan(1, 1, 4, 1, None) == B.TP_ERR_NULL
    assert B.strerror(B.TP_ERR_ALIGN).startswith("pointer")
    with pytest.raises(B.SoftmaxTpError):
        B.softmax2p_f32(None, None, -1, 1, stream=0)


CONFIGS = [(1, 4096, 4), (1024, 32768, 4), (64, 1_000_000, 4), (1, 1 << 28, 4), (4096, 21846, 2)]


def test_planner_on_the_benchmark_configurations(B):
    plans = [B.softmax_tp_plan(r, n, s) for r, n, s in CONFIGS]
    assert [p.path for p in plans] == [1, 1, 2, 2, 1]
    assert [p.launches for p in plans] == [1, 1, 2, 3, 1]
    assert plans[2].merge_kernel == 0 and plans[2].reduce.chunks <= 128  # folded by pass 2 itself
    assert plans[3].merge_kernel == 1 and plans[3].reduce.chunks > 128
    assert plans[1].rows.block == 1024                      # config 2: one workgroup per row
    assert plans[4].vector_elems == 8 and plans[4].rows.unroll <= 4
    # every algorithm has its own shape on the rows path: config 5, 2731 vectors per row
    assert (plans[4].rows.block, plans[4].rows.unroll) == (512, 2)
    assert (plans[4].rows_recompute.block, plans[4].rows_recompute.unroll) == (512, 4)
    assert (plans[4].rows_reload.block, plans[4].rows_reload.unroll) == (1024, 2)
    assert plans[3].nt_first_load == 1 and plans[2].nt_first_load == 0
    # read-only passes: two workgroups of 256 threads per CU; read-write passes: one round each
    assert (plans[3].reduce.block, plans[3].reduce.unroll, plans[3].reduce.chunks) == (256, 4, 512)
    assert (plans[3].map.block, plans[3].map.unroll, plans[3].map.chunk_vecs) == (128, 1, 256)
    assert (plans[2].map.block, plans[2].map.chunk_vecs, plans[2].reduce.chunks) == (256, 512, 8)
    for (rows, n, s), p in zip(CONFIGS, plans):
        if p.path != 2:
            continue
        nvec = -(-n // p.vector_elems)
        for shape in (p.reduce, p.map, p.mapsum):
            assert shape.chunk_vecs % (shape.block * shape.unroll) == 0
            assert shape.chunks * shape.chunk_vecs >= nvec > (shape.chunks - 1) * shape.chunk_vecs
            assert rows * shape.chunks < 2 ** 31
        most = max(p.reduce.chunks, p.mapsum.chunks)
        assert p.workspace_bytes == (2 * rows * most + 2 * rows) * 4
        assert p.workspace_bytes <= 1 << 20


def test_planner_avoids_the_merge_launch_on_short_inputs(B):
    # up to 64 MiB (16-bit: 32 MiB) a launch costs a good part of what its traffic does: at most 128
    # chunks, folded by the next pass, and larger workgroups to make up for their number
    for n, block in ((1 << 16, 256), (1 << 18, 256), (1 << 20, 256), ((1 << 20) + 1, 512), (1 << 22, 512),
                     ((1 << 22) + 1, 1024), (1 << 24, 1024)):
        p = B.softmax_tp_plan(1, n)
        assert p.path == 2 and p.reduce.chunks <= 128 and p.merge_kernel == 0 and p.launches == 2
        assert p.reduce.block == block and p.reduce.chunks * p.reduce.chunk_vecs * 4 >= n
    for n, block in ((1 << 21, 512), ((1 << 21) + 8, 1024), (1 << 24, 1024)):
        p = B.softmax_tp_plan(1, n, 2)
        assert p.reduce.chunks <= 128 and p.merge_kernel == 0 and p.reduce.block == block
    for n, s in (((1 << 24) + 1, 4), ((1 << 24) + 8, 2)):
        p = B.softmax_tp_plan(1, n, s)
        assert p.reduce.chunks > 128 and p.merge_kernel == 1 and p.launches == 3
        assert p.reduce.block == (256 if s == 4 else 512)
    B.softmax_tp_tune("block_reduce", 256)                      # an override still wins
    assert B.softmax_tp_plan(1, 1 << 23).reduce.block == 256
    B.softmax_tp_tune("block_reduce", 0)
    p = B.softmax_tp_plan(4, 1 << 24)
    assert p.reduce.chunks == 128 and p.merge_kernel == 0      # 512 workgroups over four rows
    B.softmax_tp_tune("fold_max", 64)
    assert B.softmax_tp_plan(4, 1 << 24).merge_kernel == 1
    B.softmax_tp_tune("fold_max", 0)
    with pytest.raises(B.SoftmaxTpError):
        B.softmax_tp_tune("fold_max", 5000)


def test_planner_covers_odd_shapes(B):
    rng = np.random.default_rng(3)
    for _ in range(300):
        rows = int(rng.integers(1, 5000))
        n = int(rng.integers(1, 3_000_000))
        for s, congruent in ((4, True), (4, False), (2, True), (2, False)):
            p = B.softmax_tp_plan(rows, n, s, congruent)
            V = (16 // s) if congruent else 1
            assert p.vector_elems == V
            if p.path == 1:
                assert n * s <= 256 * 1024 and p.rows.block in (4, 16, 64, 256, 512, 1024)
                nvec = -(-n // V)
                tiny, quad, wave, wave_reload = (12, 64, 352, 272) if s == 4 else (16, 128, 512, 304)
                assert (p.rows.block == 4) == (nvec <= tiny)            # tiny rows: a quad of lanes each
                assert (p.rows.block == 16) == (tiny < nvec <= quad)    # very short rows: 16 lanes each
                assert (p.rows.block == 64) == (quad < nvec <= wave)    # short rows: a wave each
                assert (p.rows_recompute.block < 256) == (nvec <= wave)
                assert (p.rows_reload.block < 256) == (nvec <= wave_reload)
                for shape in (p.rows, p.rows_recompute, p.rows_reload):
                    if shape.block < 256:   # as many loads in flight as the row has rounds, four at most
                        assert shape.unroll == min(4, -(-nvec // shape.block))
                    else:
                        assert shape.block in (256, 512, 1024) and shape.unroll in ((2, 4, 8) if s == 4 else (2, 4))
                    assert shape.chunks == 1 and shape.chunk_vecs == 0
                # the lane groups are the same for every algorithm, but the reloading variant moves to
                # the wave at 64 vectors in every format
                assert p.rows_recompute.block == p.rows.block or p.rows.block >= 256
                if p.rows_reload.block < 256:
                    wave_early = s == 2 and 64 < nvec <= 128
                    assert p.rows_reload.block == (64 if wave_early else p.rows.block)
                if p.rows.block >= 256:
                    # a lane sees at least one and at most 32 rounds of loads (element-wise 16-bit rows)
                    assert 1 <= -(-nvec // (p.rows.block * p.rows.unroll)) <= 32
            else:
                nvec = -(-n // V)
                for shape in (p.reduce, p.map, p.mapsum):
                    assert shape.chunks * shape.chunk_vecs >= nvec
    # rows of a few elements: one lane each; vectors only where every row can start on a 16-byte boundary
    for s, most, V in ((4, 9, 4), (2, 16, 8)):
        for n in range(1, most + 3):
            p = B.softmax_tp_plan(100_000, n, s)
            if n > most:
                assert p.rows.block == 4 and p.vector_elems == V
            elif n % V == 0:
                assert (p.rows.block, p.rows.unroll, p.vector_elems) == (1, n // V, V)
            else:
                assert (p.rows.block, p.rows.unroll, p.vector_elems) == (1, 2 if n <= 3 else 4, 1)
            assert p.rows_recompute.block == p.rows.block and p.rows_reload.block == p.rows.block
            q = B.softmax_tp_plan(100_000, n, s, False)
            assert q.vector_elems == 1 and (q.rows.block == 1 if n <= most else q.rows.block in (4, 16))
    assert B.softmax_tp_plan(0, 5).path == 0 and B.softmax_tp_plan(5, 0).path == 0
    big = B.softmax_tp_plan(1, 1 << 40)
    assert big.path == 2 and big.map.chunks * big.map.chunk_vecs >= (1 << 38)
    # a launch holds fewer than 2^32 threads: shapes beyond that are refused, not truncated
    assert big.map.chunks * big.map.block < 2 ** 32 and big.map.chunk_vecs > 2048
    assert B.softmax_tp_plan(1 << 29, 64).rows.block == 4       # 2^31 threads: still one launch
    assert B.softmax_tp_plan(1 << 27, 300).rows.block == 16     # a wave each would be 2^33 threads
    assert B.softmax_tp_plan(1 << 30, 300).rows.block == 1      # ... and 16 or 4 lanes each too many
    for rows, n in ((1 << 23, 8192), (1, 1 << 60), (1 << 31, 64), (1 << 33, 8)):
        with pytest.raises(B.SoftmaxTpError) as e:
            B.softmax_tp_plan(rows, n)
        assert e.value.code == B.TP_ERR_TOO_LARGE
    assert B.softmax_tp_plan(1 << 21, 8192).path == 1


def test_tuning_keys(B):
    for key in B.TUNE_KEYS:
        B.softmax_tp_tune(key, 0)
    B.softmax_tp_tune("path", 2)
    assert B.softmax_tp_plan(1024, 32768).path == 2
    B.softmax_tp_tune("path", 1)
    assert B.softmax_tp_plan(64, 60_000).path == 1
    B.softmax_tp_tune("path", 0)
    B.softmax_tp_tune("block_map", 256)
    B.softmax_tp_tune("unroll_map", 8)
    B.softmax_tp_tune("tiles_map", 3)
    p = B.softmax_tp_plan(2, 10_000_000)
    assert (p.map.block, p.map.unroll, p.map.chunk_vecs) == (256, 8, 3 * 256 * 8)
    with pytest.raises(B.SoftmaxTpError):          # bf16 keeps at most 4 loads in flight
        B.softmax_tp_plan(2, 10_000_000, 2)
    for key, bad in (("block_map", 300), ("unroll_map", 3), ("unroll_rows", 5), ("block_rows", 32), ("path", 7), ("no_such_key", 1),
                     ("direction", 3)):
        with pytest.raises(B.SoftmaxTpError):
            B.softmax_tp_tune(key, bad)
    B.softmax_tp_tune_reset()
    assert B.softmax_tp_plan(2, 10_000_000).map.block == 256     # short arrays: smaller workgroups
    assert B.softmax_tp_plan(1, 1 << 28).map.block == 128


def test_retuning_while_another_thread_plans(B):
    """softmax_tp_tune from one thread while others plan: every plan is one a single setting would
    give (the settings are read under a lock), nothing crashes."""
    import threading
    stop = threading.Event()
    seen, errors = set(), []

    def planner():
        try:
            while not stop.is_set():
                p = B.softmax_tp_plan(2, 10_000_000)
                seen.add((p.map.block, p.map.unroll))
        except Exception as e:   # noqa: BLE001
            errors.append(e)

    threads = [threading.Thread(target=planner) for _ in range(3)]
    for t in threads:
        t.start()
    try:
        for i in range(3000):
            B.softmax_tp_tune("block_map", (256, 512, 1024)[i % 3])
            B.softmax_tp_tune("unroll_map", (2, 4)[i % 2])
    finally:
        stop.set()
        for t in threads:
            t.join()
        B.softmax_tp_tune_reset()
    assert not errors
    assert seen and seen <= {(b, u) for b in (256, 512, 1024) for u in (2, 4)}


def test_constants_header_is_what_the_generator_writes(tmp_path):
    csrc = os.path.join(ROOT, "paper_2001_04438_amd", "csrc")
    committed = open(os.path.join(csrc, "expconst.h")).read()
    out_path = tmp_path / "expconst.h"
    out = subprocess.run([sys.executable, os.path.join(csrc, "gen_expconst.py"), str(out_path)],
                         check=True, capture_output=True, text=True).stdout
    assert out.strip() == committed.strip()
    assert out_path.read_text().strip() == committed.strip()
    assert open(os.path.join(csrc, "expconst.h")).read() == committed     # the tracked file is not touched


def test_fp32_extexp_accuracy_on_the_host(tmp_path):
    """Section 6.3 states a maximum error under 2 ULP over all valid inputs.  The kernel's
    evaluator header is compiled with gcc (fmaf / rintf are exact on the host too) and swept
    against 80-bit expl: every 9th fp32 value in [-104, 89] by default, every value with
    TP_EXHAUSTIVE=1 (about 80 s on 8 cores; last full run: 2,237,668,968 inputs, max 1.916 ULP)."""
    exe = tmp_path / "sweep"
    subprocess.run(["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-mfma", "-o", str(exe),
                    os.path.join(ROOT, "tests", "host_extexp_sweep.c"), "-lm", "-lpthread"], check=True)
    stride = "1" if os.environ.get("TP_EXHAUSTIVE") == "1" else "9"
    threads = str(min(16, os.cpu_count() or 1))
    out = subprocess.run([str(exe), "-104", "89", stride, threads, "4"], check=True,
                         capture_output=True, text=True).stdout.split()
    count, max_ulp, min_m, max_m, bad_n = int(out[0]), float(out[1]), float(out[2]), float(out[3]), int(out[4])
    assert count > 2.2e9 / int(stride) * 0.99
    assert max_ulp < 2.0, out
    assert bad_n == 0
    # Section 4: m = e^t with t in [-ln2/2, ln2/2], up to the slop of rounding x log2(e)
    assert math.sqrt(2) / 2 * (1 - 1e-5) <= min_m and max_m <= math.sqrt(2) * (1 + 1e-5)
    # beyond the valid range of a plain fp32 exp the pair is still exact to a few ULP
    out = subprocess.run([str(exe), "-100000", "100000", "4001", threads], check=True,
                         capture_output=True, text=True).stdout.split()
    assert int(out[4]) == 0 and 0.70 < float(out[2]) and float(out[3]) < 1.43


def test_integer_exponent_evaluator_on_the_host(tmp_path):
    """The evaluator of the 16-bit storage formats (exponent read from the bit pattern of the
    rounded sum, one-constant reduction), swept the same way: n from the bits equals
    z - 1.5 * 2^23 and round(x log2 e) everywhere up to |x| = 2.9e6; against what it approximates by
    design, e^(x - n fl(ln 2)) 2^n, it is as accurate as Algorithm 4 (< 2 ULP); against e^x itself
    the one-constant reduction costs |n| * 1.9e-9, i.e. < 5.5 ULP where fp32 exp is finite.  Every 9th
    input by default, every input with TP_EXHAUSTIVE=1 (two minutes on 8 cores; last full run:
    2,237,668,968 inputs, 1.745 ULP and 5.053 ULP, no exception in n)."""
    exe = tmp_path / "sweep"
    subprocess.run(["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-mfma", "-o", str(exe),
                    os.path.join(ROOT, "tests", "host_extexp_sweep.c"), "-lm", "-lpthread"], check=True)
    threads = str(min(16, os.cpu_count() or 1))
    stride = "1" if os.environ.get("TP_EXHAUSTIVE") == "1" else "9"
    out = subprocess.run([str(exe), "-104", "89", stride, threads, "2", "1"], check=True,
                         capture_output=True, text=True).stdout.split()
    assert int(out[0]) > 2.2e9 / int(stride) * 0.99
    assert float(out[1]) < 2.0 and int(out[4]) == 0, out
    assert 2.0 < float(out[6]) < 5.5, out           # the dropped term is visible, and bounded
    assert math.sqrt(2) / 2 * (1 - 1e-5) <= float(out[2]) and float(out[3]) <= math.sqrt(2) * (1 + 1e-5)
    for lo, hi, stride in (("-100000", "100000", "4001"), ("-2900000", "2900000", "40001")):
        out = subprocess.run([str(exe), lo, hi, stride, threads, "0", "1"], check=True,
                             capture_output=True, text=True).stdout.split()
        assert int(out[4]) == 0 and 0.69 < float(out[2]) and float(out[3]) < 1.45, out


def test_header_is_plain_c_and_cxx(tmp_path):
    """include/softmax_tp.h must be usable from C and from C++ without any HIP header, and a C
    program must link against the built library through it."""
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    inc = os.path.join(root, "include")
    lib_dir = os.path.join(root, "paper_2001_04438_amd")
    src = tmp_path / "use_header.c"
    src.write_text(
        '#include "softmax_tp.h"\n#include <stdio.h>\n'
        "int main(void) {\n"
        "    softmax_tp_plan_t p;\n"
        "    int rc = softmax_tp_plan(1, 268435456, 4, 1, &p);\n"
        '    printf("%d %d %d %d\\n", rc, p.path, p.launches, softmax2p_f32(0, 0, 0, 5, 0));\n'
        '    printf("%s\\n", softmax_tp_strerror(TP_ERR_ALIGN));\n'
        "    return rc;\n}\n")
    for compiler, std in (("gcc", "-std=c99"), ("g++", "-std=c++11")):
        subprocess.run([compiler, std, "-Wall", "-Wextra", "-Werror", "-pedantic", "-fsyntax-only", "-x",
                        "c" if compiler == "gcc" else "c++", "-I", inc, str(src)], check=True)
    exe = tmp_path / "use_header"
    subprocess.run(["gcc", "-std=c99", "-I", inc, "-o", str(exe), str(src), "-L", lib_dir,
                    "-l:libsoftmax_tp.so", "-Wl,-rpath," + lib_dir], check=True)
    out = subprocess.run([str(exe)], capture_output=True, text=True, check=True).stdout.split("\n")
    assert out[0] == "0 2 3 0" and out[1].startswith("pointer")


def test_prof_summary_cuts_a_counter_file_into_variants(tmp_path, monkeypatch):
    """prof_summary on a hand-made rocprofv3 counter file: dispatches are attributed to the variant
    whose marker kernel precedes them, bytes come from the request-size counters, VALU per element
    from SQ_INSTS_VALU."""
    from paper_2001_04438_amd import prof_summary as P
    head = ('"Correlation_Id","Dispatch_Id","Agent_Id","Queue_Id","Process_Id","Thread_Id","Grid_Size","Kernel_Id",'
            '"Kernel_Name","Workgroup_Size","LDS_Block_Size","Scratch_Size","VGPR_Count","Accum_VGPR_Count",'
            '"SGPR_Count","Counter_Name","Counter_Value","Start_Timestamp","End_Timestamp"\n')
    marker = "void tp::extexp_kernel<false>(float const*, float*, float*, long)"
    two = "void tp::rows_2p<tp::F32x4, 1024, 8>(tp::F32x4::elem const*, tp::F32x4::elem*, long)"
    mx = "void tp::chunk_max<tp::F32x4, 256, 4, false>(tp::F32x4::elem const*, tp::ChunkArgs, float*)"

    def rows(disp, kernel, counters):
        return "".join(f'{disp},{disp},"Agent 1",1,1,1,4096,7,"{kernel}",256,0,0,32,0,16,"{c}",{v},{1000 * disp},{1000 * disp + 500}\n'
                       for c, v in counters.items())

    def run(kind, per_kernel):
        d = tmp_path / f"cfg2.{kind}" / "host"
        d.mkdir(parents=True)
        text, disp = head, 0
        for variant, kernel in (("softmax2p", two), ("softmax3p_recompute", mx)):
            disp += 1
            text += rows(disp, marker, {k: 0 for k in per_kernel(marker)})
            for _ in range(2):                       # two calls per variant
                disp += 1
                text += rows(disp, kernel, per_kernel(kernel))
        (d / "1_counter_collection.csv").write_text(text)
        (tmp_path / f"cfg2.{kind}.json").write_text(json.dumps(
            {"workload": "cfg2", "rows": 4, "n": 1024, "dtype": "f32", "calls": 2,
             "variants": ["softmax2p", "softmax3p_recompute"], "ms_per_call": {}}) + "\n")

    import json
    run("rd", lambda k: {"TCC_EA0_RDREQ_sum": 10, "TCC_EA0_RDREQ_32B_sum": 2, "TCC_EA0_RDREQ_64B_sum": 3,
                         "TCC_EA0_RDREQ_128B_sum": 5 if k == two else 50})
    run("wr", lambda k: {"WRITE_SIZE": 16 if k == two else 0})
    run("sq", lambda k: {"SQ_INSTS_VALU": 640 if k == two else 64, "SQ_WAVES": 64})
    data = P.collect(str(tmp_path))
    assert list(data) == ["cfg2"] and list(data["cfg2"]["variants"]) == ["softmax2p", "softmax3p_recompute"]
    c = P.build_counters(data, "abc1234", str(tmp_path))
    two_rec = c["workloads"]["cfg2"]["softmax2p"]
    assert two_rec["fetch_bytes"] == 32 * 2 + 64 * 3 + 128 * 5 and two_rec["write_bytes"] == 16 * 1024
    assert two_rec["hbm_bytes"] == two_rec["fetch_bytes"] + two_rec["write_bytes"]
    k = two_rec["kernels"]["rows_2p"]
    assert k["launches_per_call"] == 1.0 and k["valu_lane_ops_per_element"] == 640 * 64 / 4096
    assert k["instantiation"] == "rows_2p<F32x4, 1024, 8>"
    rec = c["workloads"]["cfg2"]["softmax3p_recompute"]
    assert rec["fetch_bytes"] == 32 * 2 + 64 * 3 + 128 * 50 and rec["write_bytes"] == 0
    assert c["_meta"]["commit"] == "abc1234"
    assert P.short(two) == "rows_2p<F32x4, 1024, 8>" and P.base(mx) == "chunk_max"


def test_bench_line_never_prints_an_unlabelled_fraction_above_one():
    """bench.describe_variant: with a counter record a cache-assisted variant is priced on the bytes
    that reached memory; without one, a rate above the HBM peak is withheld and explained."""
    sys.path.insert(0, ROOT)
    import bench
    alg = 3 * 1024 * 32768 * 4                       # Two-Pass on 1024 x 32768 fp32
    copy_ms, copy_bytes = 0.046, 2 * 1024 * 32768 * 4
    e = bench.describe_variant({}, alg, 0.045, copy_ms, copy_bytes, {"hbm_bytes": 260_000_000})
    assert e["cache_assisted"] is True and e["hbm_bytes_measured"] == 260_000_000
    assert e["GBps_algorithmic"] > bench.HBM_PEAK_GBS > e["GBps_effective"]
    assert 0 < e["frac_of_hbm_peak"] <= 1 and e["frac_of_hbm_peak"] == pytest.approx(260e6 / 0.045 / 1e6 / 8000)
    assert e["frac_of_stream_copy"] == pytest.approx((260e6 / 0.045) / (copy_bytes / copy_ms))
    e = bench.describe_variant({}, alg, 0.045, copy_ms, copy_bytes, None)
    assert e["cache_assisted"] is None and e["frac_of_hbm_peak"] is None and "frac_of_hbm_peak_note" in e
    e = bench.describe_variant({}, alg, 0.060, copy_ms, copy_bytes, {"hbm_bytes": alg})
    assert e["cache_assisted"] is False and e["frac_of_hbm_peak"] == pytest.approx(alg / 0.060 / 1e6 / 8000)


def test_bench_refuses_more_than_one_gpu():
    """Everything here runs on one GPU: asked for more, bench.py says so and exits before any GPU work."""
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                         capture_output=True, text=True, timeout=120)
    assert res.returncode != 0
    assert "one GPU" in res.stderr and res.stdout.strip() == ""
