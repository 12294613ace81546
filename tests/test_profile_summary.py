"""The helper that turns rocprofv3 counter output into profiles/traffic_*.txt: scaling by the
calibration copy, the per-kernel means, and the source fingerprint bench.py checks."""

import os

from paper_2407_17678_amd import profile_summary as P

HEAD = "Correlation_Id,Dispatch_Id,Agent_Id,Queue_Id,Process_Id,Thread_Id,Grid_Size,Kernel_Id,Kernel_Name,Workgroup_Size,LDS_Block_Size,Scratch_Size,VGPR_Count,Accum_VGPR_Count,SGPR_Count,Counter_Name,Counter_Value,Start_Timestamp,End_Timestamp\n"


def _row(kernel, counter, value):
    return '1,1,1,1,1,1,1,1,"%s",256,0,0,0,0,0,%s,%s,0,1\n' % (kernel, counter, value)


def test_traffic_is_scaled_by_the_largest_copy(tmp_path):
    k = "void s2::(anonymous namespace)::fwd_pipe_kernel<128, false>(s2::AttnParams)"
    f, w = tmp_path / "f.csv", tmp_path / "w.csv"
    # FETCH_SIZE reads half the KiB the 1 GiB copy moved (factor 2), WRITE_SIZE all of them (factor 1)
    f.write_text(HEAD + _row("__amd_rocclr_copyBuffer", "FETCH_SIZE", 524288) + _row("__amd_rocclr_copyBuffer", "FETCH_SIZE", 100)
                 + _row(k, "FETCH_SIZE", 1000) + _row(k, "FETCH_SIZE", 3000))
    w.write_text(HEAD + _row("__amd_rocclr_copyBuffer", "WRITE_SIZE", 1048576) + _row(k, "WRITE_SIZE", 500))
    text = P.traffic("7b_32k", str(f), str(w))
    lines = text.splitlines()
    assert lines[0] == "# sources " + P.source_fingerprint()
    row = [l for l in lines if l.startswith("fwd_pipe_kernel ")][0].split()
    assert int(row[1]) == 2000 * 2 * 1024 + 500 * 1024     # mean fetch x 2, write x 1, KiB -> bytes


def test_fingerprint_follows_the_kernel_sources():
    a = P.source_fingerprint()
    assert a == P.source_fingerprint() and len(a) == 16
    # every committed traffic summary either carries a fingerprint line or is refused by bench.py
    prof = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(P.__file__))), "profiles")
    for name in os.listdir(prof):
        if name.startswith("traffic_") and name.endswith(".txt"):
            with open(os.path.join(prof, name)) as fh:
                assert fh.readline().startswith("# sources "), name


def test_the_ds_keeping_dkdv_instantiation_is_told_apart(tmp_path):
    plain = "void s2::(anonymous namespace)::dkdv_kernel<128, false, 64, false, false>(s2::AttnParams)"
    keeps = "void s2::(anonymous namespace)::dkdv_kernel<128, false, 64, false, true>(s2::AttnParams)"
    f, w = tmp_path / "f.csv", tmp_path / "w.csv"
    copy = "__amd_rocclr_copyBuffer"
    f.write_text(HEAD + _row(copy, "FETCH_SIZE", 524288) + _row(plain, "FETCH_SIZE", 1000) + _row(keeps, "FETCH_SIZE", 2000))
    w.write_text(HEAD + _row(copy, "WRITE_SIZE", 1048576) + _row(plain, "WRITE_SIZE", 10) + _row(keeps, "WRITE_SIZE", 4000))
    rows = {l.split()[0]: int(l.split()[1]) for l in P.traffic("7b_32k", str(f), str(w)).splitlines() if not l.startswith("#")}
    assert rows == {"dkdv_kernel": (2000 + 10) * 1024, "dkdv_kernel_keeping_ds": (4000 + 4000) * 1024}
