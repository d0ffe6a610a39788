"""Thin Python binding of libflare_rates.so (see include/flare_rates.h): machine-rate micro-benchmarks.

Argument marshalling and the list of runs only; every measurement is a kernel of the library.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libflare_rates.so")
EXPORTS = ["flare_rates_count", "flare_rates_name", "flare_rates_scratch_bytes", "flare_rates_run"]
NOMINAL_GHZ = 2.4


class RatesResult(ctypes.Structure):
    _fields_ = [("ms", ctypes.c_double), ("vector_ops", ctypes.c_double), ("matrix_ops", ctypes.c_double),
                ("bytes", ctypes.c_double), ("shader_mhz", ctypes.c_double)]


_lib = None


def load():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libflare_rates.so not found: run `python -m paper_2508_12594_amd.build`")
        lib = ctypes.CDLL(LIB_PATH)
        lib.flare_rates_count.restype = ctypes.c_int
        lib.flare_rates_name.restype = ctypes.c_char_p
        lib.flare_rates_name.argtypes = [ctypes.c_int]
        lib.flare_rates_scratch_bytes.restype = ctypes.c_size_t
        lib.flare_rates_run.restype = ctypes.c_int
        lib.flare_rates_run.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p,
                                        ctypes.c_size_t, ctypes.c_void_p, ctypes.POINTER(RatesResult)]
        _lib = lib
    return _lib


def names():
    lib = load()
    return [lib.flare_rates_name(i).decode() for i in range(lib.flare_rates_count())]


def run_all(iters=20000):
    """Every experiment at the wave counts that matter; returns a list of dict rows.

    Per row: ms, clocks per instruction and SIMD at the nominal 2.4 GHz (`clk`: duration x 2.4 GHz divided by
    the instructions one SIMD issued, vector + matrix), the shader clock the kernel itself saw, and for the copy GB/s."""
    import torch
    lib = load()
    nbytes = int(lib.flare_rates_scratch_bytes())
    scratch = torch.zeros(nbytes + 256, dtype=torch.uint8, device="cuda")
    base = (scratch.data_ptr() + 255) & ~255
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    all_names = names()
    plan = [("copy", 1, 0)]
    for op in ("v_exp_f32", "v_fma_f32", "v_cvt_pk_bf16_f32", "v_max3_f32", "v_perm_b32", "v_dot2c_f32_bf16",
               "v_add_f32", "v_mfma_f32_32x32x16_bf16", "v_mfma_f32_16x16x32_bf16"):
        for w in (1, 2, 4):
            plan.append((op, w, 0))
    rows = []

    def one(i, w, param, it):
        res = RatesResult()
        rc = lib.flare_rates_run(i, w, param, it, ctypes.c_void_p(base), ctypes.c_size_t(nbytes), stream,
                                 ctypes.byref(res))
        if rc != 0:
            raise RuntimeError("flare_rates_run(%s, waves %d, param %d) failed: %d" % (all_names[i], w, param, rc))
        ops = res.vector_ops + res.matrix_ops
        row = {"experiment": all_names[i], "waves_per_simd": w, "param": param, "ms": round(res.ms, 4),
               "vector_per_simd": res.vector_ops, "matrix_per_simd": res.matrix_ops,
               "shader_mhz": round(res.shader_mhz, 1)}
        if res.bytes:
            row["GBps"] = round(res.bytes / (res.ms * 1e-3) / 1e9, 1)
        if ops:
            row["clk_per_instr"] = round(res.ms * 1e-3 * NOMINAL_GHZ * 1e9 / ops, 2)
        row["clk_total"] = round(res.ms * 1e-3 * NOMINAL_GHZ * 1e9, 0)
        rows.append(row)

    for name, w, param in plan:
        one(all_names.index(name), w, param, iters)
    for i, n in enumerate(all_names):
        if n.startswith("same wave"):
            for w in (1, 2):
                for k in (1, 2, 4, 8, 16):
                    one(i, w, k, iters // 2)
        elif n.startswith("other wave"):
            for w in (2, 3):
                for param in (1, 2, 0):
                    one(i, w, param, iters // 4)
        elif n.startswith("softmax tile"):
            for w in (1, 2, 3):
                for k in (1, 2, 3):
                    one(i, w, k, iters // 2)
        elif n.startswith("fp64"):
            for param in (0, 1, 2, 3, 4, 8, 9, 10, 11, 12, 16, 19, 24):
                one(i, 1, param, iters)
    return rows


def derive(rows):
    """The handful of constants the roofline figures use, from the rows of run_all (2.4 GHz clocks per wave64
    instruction and SIMD unless named otherwise)."""
    def row(prefix, w, param=0):
        for r in rows:
            if r["experiment"].startswith(prefix) and r["waves_per_simd"] == w and r["param"] == param:
                return r
        return None

    out = {}
    copy = row("copy", 1)
    if copy:
        out["copy_GBps_read_plus_write"] = copy["GBps"]
    for key, name in (("exp", "v_exp_f32"), ("fma", "v_fma_f32"), ("add", "v_add_f32"), ("pack", "v_cvt_pk_bf16_f32"),
                      ("max3", "v_max3_f32"), ("perm", "v_perm_b32"), ("dot2", "v_dot2c_f32_bf16")):
        r = row(name, 2)
        if r:
            out[key + "_clk"] = r["clk_per_instr"]
    for key, name in (("mfma32", "v_mfma_f32_32x32x16_bf16"), ("mfma16", "v_mfma_f32_16x16x32_bf16")):
        r = row(name, 2)
        if r:   # the matrix pipe alone runs at a reduced clock: report both the nominal-clock figure and its own clocks
            out[key + "_pipe_clk"] = r["clk_per_instr"]
            out[key + "_pipe_own_clocks"] = round(r["clk_per_instr"] * r["shader_mhz"] / (NOMINAL_GHZ * 1e3), 1)
            out[key + "_alone_shader_mhz"] = r["shader_mhz"]
    # what one matrix instruction costs a vector stream of the same wave that alone saturates the SIMD:
    # (duration - exponentials x their own clocks) / matrix instructions, at k exponentials per matrix instruction
    e = row("v_exp_f32", 2)
    for key, prefix in (("mfma32", "same wave: 1 mfma 32x32x16 + k v_exp_f32"),
                        ("mfma16", "same wave: 1 mfma 16x16x32 + k v_exp_f32")):
        for k in (4, 8, 16):
            r = row(prefix, 2, k)
            if r and e:
                out["%s_cost_to_vector_stream_k%d" % (key, k)] = round(
                    (r["clk_total"] - r["vector_per_simd"] * e["clk_per_instr"]) / r["matrix_per_simd"], 1)
    for w in (2, 3):
        m, v, b = (row("other wave: mfma 32x32x16", w, p) for p in (1, 2, 0))
        if m and v and b:
            out["other_wave_w%d_ms_matrix_vector_both" % w] = [m["ms"], v["ms"], b["ms"]]
            out["other_wave_w%d_shader_mhz_matrix_vector_both" % w] = [m["shader_mhz"], v["shader_mhz"], b["shader_mhz"]]
    for k in (1, 2, 3):
        r = row("softmax tile", 2, k)
        if r:
            tiles = r["matrix_per_simd"] / (2 + k)
            out["tile_ns_%d_score_mfma" % k] = round(r["ms"] * 1e6 / tiles, 1)
    return out
