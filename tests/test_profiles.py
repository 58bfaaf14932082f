"""The rocprofv3 summaries under profiles/ against the byte model and the
library as built: bench.py reads its measured-traffic figure from these files,
so a summary that no longer belongs to the kernel the library launches (another
template signature), or whose algorithmic bytes disagree with the byte table,
must fail here."""
import importlib.util
import os
import re

import pytest

from paper_2012_05396_amd import binding as B
from paper_2012_05396_amd import workloads

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench():
    spec = importlib.util.spec_from_file_location("bench", os.path.join(ROOT, "bench.py"))
    m = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(m)
    return m


# bytes per element of the plain steps-delay iteration: reads K gradients,
# K local weights, pre_weight, w, momentum; writes K local weights, w, momentum
PLAIN_B_PER_ELEM = {(4, 4): 68, (8, 4): 116, (16, 4): 212, (8, 2): 100}   # (K, gradient bytes) -> B


@pytest.mark.parametrize("key", sorted(_bench().PROFILE_OF))
def test_profile_matches_byte_model_and_current_kernel(key):
    bench = _bench()
    wlname, gdname = key
    wl = workloads.workload(wlname)
    N, K = sum(workloads.numels(wl.tensors)), wl.K
    gb = 4 if gdname == "f32" else 2
    gd = {"f32": B.SSD_GRAD_F32, "bf16": B.SSD_GRAD_BF16, "f16": B.SSD_GRAD_F16}[gdname]
    p = bench.read_profile(bench.PROFILE_OF[key])
    per_elem = bench.bytes_per_element(K, 2, 0, False, gb)[1]
    assert per_elem == PLAIN_B_PER_ELEM[(K, gb)] == (8 + gb) * K + 20
    assert p["algorithmic"] == per_elem * N
    # measured HBM traffic: no wasted re-reads, and nothing missing
    assert 0.999 <= p["traffic"] / p["algorithmic"] <= 1.01
    # the summary is of the kernel this library launches for that K
    assert p["kernel"] == bench.dominant_kernel_name(B, K, gd)


def test_unfused_profile_shows_the_bytes_fusion_saves():
    text = open(os.path.join(ROOT, "profiles", "unfused_vgg16_K8_k4.txt")).read()
    got = [float(x) for x in re.findall(r"ssd_glu_kernel<0, 0> = [\d,]+ B = ([\d.]+) B per element", text)]
    assert len(got) == 2                      # one stream, two streams
    for b in got:
        assert abs(b - (20 * 8 + 16)) < 1.0   # server launch + K GLU launches: gradients read twice
    ms = [float(x) for x in re.findall(r"([\d.]+) ms per step", text)]
    assert len(ms) == 3 and ms[2] < 0.6 * min(ms[:2])   # fused vs unfused
