"""Host-side pieces of the benchmark, checked without a GPU: the algorithmic work per backward pass that the
roofline figures are priced with, the sorting of profiled kernels into the parts of a minibatch backward pass,
and that the stored counter figures belong to the kernel sources in the tree."""
import json
import os

import pytest

import bench
import bench_traffic_record as rec
import lf_inputs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_algorithmic_work_of_the_five_configurations():
    """Single sample: 4 bytes per entry of every matrix the chain reads (w^3..w^L) and every gradient written
    (nabla_w^2..nabla_w^L).  Minibatch: 2 B flops per matrix entry and contraction."""
    want = {
        "cfg1": ("hbm", 4 * 256 * 256 * (6 + 7)),
        "cfg2": ("hbm", 4 * 1024 * 1024 * (30 + 31)),
        "cfg3": ("hbm", 4 * 4096 * 4096 * (62 + 63)),
        "cfg4": ("mfma", 2 * 256 * 4096 * 4096 * (30 + 31)),
        "cfg5": ("mfma", 2 * 512 * 8192 * 8192 * (46 + 47)),
    }
    for name, (bound, work) in want.items():
        w = bench.algorithmic_work(lf_inputs.CONFIGS[name])
        assert w["bound"] == bound and w["bwd"] == work, name
        assert w["peak"] == (8000.0 if bound == "hbm" else {"cfg4": 157.3, "cfg5": 2500.0}[name])


def test_descent_step_work_reads_and_rewrites_the_weights():
    s = lf_inputs.CONFIGS["cfg2"]
    plain, stepped = bench.algorithmic_work(s), bench.algorithmic_work(s, sgd=True)
    assert stepped["bwd"] - plain["bwd"] == 4 * 1024 * 1024 * 31


@pytest.mark.parametrize("name,part", [
    ("void lf::(anonymous namespace)::big::k_gemm_big<false, true, 0>(lf::(anonymous namespace)::GemmArgs)", "chain product (bp2)"),
    ("void lf::(anonymous namespace)::big::k_gemm_big<false, false, 0>(lf::(anonymous namespace)::GemmArgs)", None),
    ("void lf::(anonymous namespace)::big::k_gemm_big<true, true, 3>(lf::(anonymous namespace)::GemmArgs)", "gradient product (bp4)"),
    ("void lf::(anonymous namespace)::big::k_grad_stream<0>(lf::(anonymous namespace)::GemmArgs, int, int)", "gradient product (bp4)"),
    ("void lf::(anonymous namespace)::k_gemm<float, false, true, 0>(lf::(anonymous namespace)::GemmArgs)", "chain product (bp2)"),
    ("void lf::(anonymous namespace)::k_gemm<float, true, true, 3>(lf::(anonymous namespace)::GemmArgs)", "gradient product (bp4)"),
    ("void lf::(anonymous namespace)::k_gemm<__bf16, false, false, 1>(lf::(anonymous namespace)::GemmArgs)", None),
    ("_ZN2lf12_GLOBAL__N_114k_split_finishIDF16bLi2EEEvPKfimiS3_PKT_PvPDF16b", "chain split finish (bp2)"),
    ("_ZN2lf12_GLOBAL__N_114k_split_finishIDF16bLi1EEEvPKfimiS3_PKT_PvPDF16b", None),
    ("void lf::(anonymous namespace)::k_split_finish<float, 2>(float const*, int, unsigned long, int)", "chain split finish (bp2)"),
    ("lf::(anonymous namespace)::k_bias_grad(float const*, float*, int, int, float)", "bias sums (bp3)"),
    ("_ZN2lf12_GLOBAL__N_114k_output_errorIDF16bEEvPKT_S4_PfPDF16bmf", "output error (bp1)"),
    ("void at::native::vectorized_elementwise_kernel<4, at::native::FillFunctor<float>>", None),
])
def test_profiled_kernels_are_sorted_into_the_parts_of_the_backward_pass(name, part):
    assert rec.backward_part(name) == part


def test_stored_counter_figures_belong_to_the_sources_in_the_tree():
    """profiles/traffic.json is quoted by bench.py only while its hashes match the kernel sources; a stale record
    would silently turn roofline.traffic into null."""
    stored = json.load(open(os.path.join(ROOT, "profiles", "traffic.json")))
    assert stored["kernel_source_sha256"] == rec.source_hash(rec.PERSISTENT_SOURCES)
    for key in ("cfg2_k8", "cfg3_k8", "cfg4_k4", "cfg5_k8"):
        cfg, k = key.split("_k")
        t = bench.measured_traffic(cfg, int(k))
        assert isinstance(t, int) and t > 0, key
        e = stored[key]
        assert t == e["fetch_bytes"] + e["write_bytes"]
        # never less than what the method must move (weights read once, gradients written once)
        spec = lf_inputs.CONFIGS[cfg]
        sizes = bench.matrix_sizes(spec)
        es = 4 if spec.dtype == "f32" else 2
        assert t >= es * sum(sizes[1:]) + 4 * sum(sizes)
    assert bench.measured_traffic("cfg1", 2) is None and bench.measured_traffic("cfg5", 3) is None


def test_the_measurement_aid_exports_what_bench_calls():
    """libbench_probe.so (built beside the library) carries the three entry points bench.py's machine rates use;
    called with bad arguments they refuse without touching a device."""
    import ctypes
    path = os.path.join(ROOT, "libbench_probe.so")
    if not os.path.exists(path):
        pytest.skip("libbench_probe.so is not built")
    p = ctypes.CDLL(path)
    for name in ("probe_stream", "probe_mfma_loop", "probe_strips_beside_rows"):
        assert hasattr(p, name), name
    p.probe_strips_beside_rows.restype = ctypes.c_double
    p.probe_strips_beside_rows.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int,
                                           ctypes.c_void_p]
    assert p.probe_strips_beside_rows(3, None, None, 1, 1, None) < 0        # no such mode
    assert p.probe_strips_beside_rows(2, None, None, 16, 62, None) < 0      # no buffers
    p.probe_stream.restype = ctypes.c_double
    p.probe_stream.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t,
                               ctypes.c_void_p, ctypes.c_void_p]
    assert p.probe_stream(0, 512, None, None, 1 << 20, None, None) == 0.0
