"""HBM copy and LDS read bandwidth that plain kernels reach on the device at hand, for putting the
replay's achieved figures into proportion.

    python -m paper_2401_08156_amd.peaks [--json]
"""
import argparse
import json

from . import binding


def measure():
    rc, rep = binding.vms_measure_peaks()
    if rc != binding.VMS_OK:
        raise binding.VmsError(rc, "vms_measure_peaks (hip error %d)" % rep.hip_error)
    return dict(compute_units=rep.compute_units, clock_mhz=rep.clock_mhz,
                hbm_copy_gbs=rep.hbm_copy_gbs, copy_ms=rep.copy_ms, copy_bytes=rep.copy_bytes,
                lds_read_gbs=rep.lds_read_gbs, lds_ms=rep.lds_ms, lds_bytes=rep.lds_bytes,
                hbm_read_gbs=rep.hbm_read_gbs, read_ms=rep.read_ms, read_bytes=rep.read_bytes)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--json", action="store_true")
    args = ap.parse_args()
    m = measure()
    if args.json:
        print(json.dumps(m))
        return
    print("compute units %d, clock %d MHz" % (m["compute_units"], m["clock_mhz"]))
    print("copy kernel, 1 GiB read + 1 GiB written: %.3f ms, %.0f GB/s" % (m["copy_ms"], m["hbm_copy_gbs"]))
    print("read-only kernel, 1 GiB read: %.3f ms, %.0f GB/s" % (m["read_ms"], m["hbm_read_gbs"]))
    print("LDS read loop, 16 B per lane and trip, all compute units: %.3f ms, %.0f GB/s" % (m["lds_ms"], m["lds_read_gbs"]))


if __name__ == "__main__":
    main()
