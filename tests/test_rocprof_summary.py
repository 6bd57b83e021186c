"""The profile summariser's selection of the timed launches, on a synthetic trace (no GPU, no rocprofv3)."""
import csv

from paper_2512_09685_amd import rocprof_summary as rs


def write_trace(path, kernels):
    with open(path, "w", newline="") as f:
        w = csv.writer(f, quoting=csv.QUOTE_ALL)
        w.writerow(["Kind", "Kernel_Name", "Start_Timestamp", "End_Timestamp"])
        t = 1000
        for name, dur_ns in kernels:
            w.writerow(["KERNEL_DISPATCH", name, t, t + dur_ns])
            t += dur_ns + 50


def test_timed_launches_are_counted_back_from_the_end(tmp_path):
    main = "void star::aff_mfma_kernel<16, star::RowF32, true, false>(float*, float*)"
    small = "star::reduce_kernel(double const*, int, double*, float*)"
    other = "__amd_rocclr_copyBuffer"
    seq = [(other, 500)]
    # 7 slow wake-up / warm-up calls, 4 timed calls, 2 first-call samples; every call = main kernel + 2 small ones
    for dur in [1900] * 7 + [1500, 1510, 1490, 1500] + [1700, 1720]:
        seq += [(main, dur * 1000), (small, 4000), (small, 5000)]
    p = tmp_path / "trace.csv"
    write_trace(p, seq)
    disp = rs.dispatches(str(p))
    assert len(disp) == 13 * 3 and all("star::" in k for k, _ in disp)          # the copy kernel is not the library's
    name, sel, total = rs.timed_only(disp, timed=4, after=2)
    assert name == "star::aff_mfma_kernel<16, star::RowF32, true, false>"
    assert sel[name] == [1500.0, 1510.0, 1490.0, 1500.0]                          # microseconds, the timed four only
    assert sel["star::reduce_kernel"] == [4.0, 5.0] * 4                           # two per call, the same calls
    assert total[name] == 13


def test_counter_values_group_by_kernel(tmp_path):
    p = tmp_path / "c.csv"
    with open(p, "w", newline="") as f:
        w = csv.writer(f, quoting=csv.QUOTE_ALL)
        w.writerow(["Kernel_Name", "Counter_Name", "Counter_Value"])
        w.writerow(["void star::aff_kernel<8, star::RowF32, true, false>(float*)", "FETCH_SIZE", 10.0])
        w.writerow(["void star::aff_kernel<8, star::RowF32, true, false>(float*)", "WRITE_SIZE", 3.0])
        w.writerow(["void star::aff_kernel<8, star::RowF32, true, false>(float*)", "FETCH_SIZE", 12.0])
        w.writerow(["__amd_rocclr_copyBuffer", "FETCH_SIZE", 524307.8])
    v = rs.counter_values(str(p), "FETCH_SIZE")
    assert v["star::aff_kernel<8, star::RowF32, true, false>"] == [10.0, 12.0]
    assert v["__amd_rocclr_copyBuffer"] == [524307.8]
