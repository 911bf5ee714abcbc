"""Thin ctypes binding and driver of libtva_ubench (include/tva_ubench.h): the microbenchmarks of the
MI355X rates the attention kernels are priced against.  Measurement aid only; nothing on the hot path
imports it.  `bench.py --microbench` prints what `run_all` returns."""
from __future__ import annotations

import ctypes
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtva_ubench.so")
SRC_PATH = os.path.join(_HERE, "csrc", "ubench.hip")
INCLUDE_DIR = os.path.join(os.path.dirname(_HERE), "include")
EXPORTS = ("tva_ubench_mfma_valu", "tva_ubench_lds", "tva_ubench_stream", "tva_ubench_empty", "tva_ubench_valu_attn", "tva_ubench_reread")
_lib = None


def build_library(verbose: bool = False) -> str:
    from .binding import HIPCC_FLAGS
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, "-I", INCLUDE_DIR, "-shared", "-fPIC", "-o", LIB_PATH, SRC_PATH]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    lines = [l for l in res.stdout.splitlines() if "is not a recognized feature" not in l]
    if verbose or res.returncode:
        print("\n".join(lines))
    if res.returncode:
        raise RuntimeError("hipcc failed building libtva_ubench.so")
    return LIB_PATH


def load_library():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
        import torch  # noqa: F401  (one HIP runtime per process: torch's)
        lib = ctypes.CDLL(LIB_PATH)
        i32, vp = ctypes.c_int32, ctypes.c_void_p
        lib.tva_ubench_mfma_valu.argtypes = [i32, i32, i32, i32, i32, i32, vp, vp, vp]
        lib.tva_ubench_lds.argtypes = [i32, i32, i32, i32, vp, vp, vp]
        lib.tva_ubench_stream.argtypes = [i32, vp, ctypes.c_size_t, i32, vp, vp]
        lib.tva_ubench_empty.argtypes = [vp]
        lib.tva_ubench_reread.argtypes = [i32, vp, ctypes.c_size_t, i32, i32, vp, vp]
        lib.tva_ubench_valu_attn.argtypes = [vp, vp]      # (tva_ubench_attn_args *, stream): paper_2510_26577_amd/small_rows.py
        _lib = lib
    return _lib


def run_all(n_cu: int = 256):
    """Runs every probe on cuda:0; returns a dict of plain numbers (cycles are shader-clock cycles of the
    slowest wave; `ghz` is the clock the probe ran at, from the 100 MHz counter)."""
    import torch
    lib = load_library()
    dev = "cuda:0"
    st = torch.cuda.current_stream()
    sp = ctypes.c_void_p(st.cuda_stream)
    sink = torch.zeros(512, dtype=torch.float32, device=dev)
    res = {}

    def timed_waves(call, workgroups, waves_per_simd, iters):
        waves = workgroups * 4 * waves_per_simd
        out = torch.zeros(2 * waves, dtype=torch.int64, device=dev)
        for _ in range(2):                                   # first run warms the clocks and the code cache
            rc = call(out)
            assert rc == 0, rc
            torch.cuda.synchronize()
        o = out.cpu().numpy().reshape(waves, 2)
        cyc, ticks = float(o[:, 0].max()), float(o[:, 1].max())
        return cyc / iters, (cyc / (ticks / 100e6)) / 1e9 if ticks > 0 else 0.0

    # ---- matrix instruction alone, and with vector work behind each one ----
    iters = 4000
    mf = {}
    for wps in (1, 2):
        for nacc, k, e in [(1, 0, 0), (4, 0, 0), (4, 2, 0), (4, 4, 0), (4, 6, 0), (4, 8, 0), (4, 10, 0), (4, 12, 0),
                           (4, 16, 0), (4, 0, 1), (4, 0, 2), (4, 0, 4), (4, 3, 2), (4, 5, 2), (0, 8, 0), (0, 0, 8)]:
            per_iter, ghz = timed_waves(
                lambda out: lib.tva_ubench_mfma_valu(nacc, k, e, wps, n_cu, iters, out.data_ptr(), sink.data_ptr(), sp),
                n_cu, wps, iters)
            groups = max(nacc, 1)
            mf[f"waves_per_simd={wps} mfma_accs={nacc} fma={k} exp={e}"] = {
                "cycles_per_group": per_iter / groups, "ghz": ghz}
    res["mfma_valu"] = mf
    base = mf["waves_per_simd=1 mfma_accs=4 fma=0 exp=0"]
    # 32x32x16 MFMA = 32768 flop per wave; 4 SIMDs per CU
    res["mfma_tflops_at_measured_rate"] = 32768 * 4 * n_cu * base["ghz"] * 1e9 / base["cycles_per_group"] / 1e12

    # ---- LDS reads ----
    lds = {}
    for tr in (0, 1):
        for wps in (1, 2):
            per_iter, ghz = timed_waves(
                lambda out: lib.tva_ubench_lds(tr, wps, n_cu, 2000, out.data_ptr(), sink.data_ptr(), sp), n_cu, wps, 2000)
            # per iteration every lane reads 128 bytes; 256 * wps lanes per CU
            lds[f"{'ds_read_b64_tr_b16' if tr else 'ds_read_b128'} waves_per_simd={wps}"] = {
                "bytes_per_clk_per_cu": 128 * 256 * wps / per_iter, "ghz": ghz}
    res["lds"] = lds

    # ---- streaming read of 1 GiB (larger than the 256 MB last-level cache) ----
    nbytes = 1 << 30
    buf = torch.empty(nbytes // 4, dtype=torch.int32, device=dev)
    buf.random_(0, 1 << 20)
    stream = {}
    for to_lds in (0, 1, 2):
        for wgs in (n_cu * 4, n_cu * 8, n_cu * 16):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            best = 1e30
            for _ in range(5):
                e0.record(st)
                rc = lib.tva_ubench_stream(to_lds, buf.data_ptr(), nbytes, wgs, sink.data_ptr(), sp)
                assert rc == 0, rc
                e1.record(st)
                torch.cuda.synchronize()
                best = min(best, e0.elapsed_time(e1))
            name = ("global_load nt", "global_load_lds", "global_load_lds nt")[to_lds]
            stream[f"{name} workgroups={wgs}"] = {"GB_per_s": nbytes / best / 1e6}
    res["stream_read_1GiB"] = stream
    del buf

    # ---- L2 -> CU: every workgroup re-reads 1 MiB (it stays in the L2 of each XCD), one workgroup per CU ----
    small = torch.empty((1 << 20) // 4, dtype=torch.int32, device=dev)
    small.random_(0, 1 << 20)
    l2 = {}
    for to_lds in (0, 1):
        for wgs in (n_cu // 2, n_cu, 2 * n_cu):
            reps = 64
            best = 1e30
            for _ in range(4):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(st)
                rc = lib.tva_ubench_reread(to_lds, small.data_ptr(), 1 << 20, reps, wgs, sink.data_ptr(), sp)
                assert rc == 0, rc
                e1.record(st)
                torch.cuda.synchronize()
                best = min(best, e0.elapsed_time(e1))
            total = wgs * reps * (1 << 20)
            l2[f"{'global_load_lds' if to_lds else 'global_load'} workgroups={wgs}"] = {
                "TB_per_s": total / best / 1e9, "GB_per_s_per_workgroup": total / best / 1e6 / wgs}
    res["l2_reread_1MiB"] = l2
    del small

    # ---- empty kernel: back-to-back launches replayed from one graph ----
    n = 200
    g = torch.cuda.CUDAGraph()
    s2 = torch.cuda.Stream()
    lib.tva_ubench_empty(ctypes.c_void_p(s2.cuda_stream))
    torch.cuda.synchronize()
    with torch.cuda.graph(g, stream=s2):
        for _ in range(n):
            lib.tva_ubench_empty(ctypes.c_void_p(s2.cuda_stream))
    best = 1e30
    with torch.cuda.stream(s2):
        for _ in range(5):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(s2)
            g.replay()
            e1.record(s2)
            torch.cuda.synchronize()
            best = min(best, e0.elapsed_time(e1))
    res["empty_kernel_us_per_launch_in_graph"] = best * 1e3 / n
    return res
