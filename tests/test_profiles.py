"""The measurement records under profiles/ belong to the kernel sources in the tree: the traffic
record names a digest of csrc/ (bench.py reports no traffic figure when it does not match), every
summary gives the command that made it, and nothing under profiles/ is runnable or raw output."""
import hashlib
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PROFILES = os.path.join(ROOT, "profiles")
CSRC = os.path.join(ROOT, "paper_2603_10026_amd", "csrc")


def csrc_digest():
    h = hashlib.sha256()
    for name in sorted(os.listdir(CSRC)):
        h.update(name.encode())
        with open(os.path.join(CSRC, name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def test_traffic_record_was_measured_on_the_kernel_sources_in_the_tree():
    text = open(os.path.join(PROFILES, "bench_all_workloads_hbm_traffic.txt")).read()
    m = re.search(r"^SOURCES (\w+)$", text, re.M)
    assert m, "the traffic record names the sources it was measured on"
    assert m.group(1) == csrc_digest(), (
        "profiles/ was measured on other kernel sources: regenerate the summaries "
        "(the commands are in their headers) after changing anything under csrc/")
    labels = re.findall(r"^TRAFFIC (\S+) (\d+) (\d+)$", text, re.M)
    assert {"w1_softmax", "w2_attention_prefill", "w3_decode_splitk", "w4_rmsnorm_gemm"} <= {l[0] for l in labels}


def test_profiles_hold_short_text_summaries_with_their_commands():
    names = sorted(os.listdir(PROFILES))
    assert names, "profiles/ is not empty"
    for name in names:
        path = os.path.join(PROFILES, name)
        assert name.endswith((".txt", ".md")), name
        assert os.path.getsize(path) < 64 * 1024, name
        text = open(path).read()
        assert "command" in text, f"{name} gives the command that made it"
        assert "_work/" not in text, f"{name}: its command runs committed files only"
