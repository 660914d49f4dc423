"""Random-row yardsticks of the GPU this runs on.  Gather (bp_gather_calibration): how fast rows of 64 .. 512 bytes
come out of a table far larger than the caches when nothing else runs, with 1 / 2 / 4 / 8 rows in flight per lane
group: the ceiling any kernel that gathers rows of that size can reach.  Scatter (bp_scatter_calibration): how fast
every row of a table is written once, in a random order and in ascending order, with nothing read but the order: the
ceiling of a forward pass over one-lookup bags, which writes one output row per lookup.  Prints two tables.

    python -m paper_2202_12429_amd.gather_yardstick
"""
import math

import torch

import paper_2202_12429_amd as bp


def median_us(launch, launches=12):
    """Median duration of `launches` launches by the library's own event brackets (the kernel's begin and end, as for
    the kernels of a training step), after one launch that is not counted."""
    launch(0)
    torch.cuda.synchronize()
    bp.bp_profile_select(["copy_calibration"])
    bp.bp_profile_enable(True)
    for k in range(launches):
        launch(k)
    torch.cuda.synchronize()
    bp.bp_profile_collect()
    med = bp.profile_spread("copy_calibration")[1] * 1e3
    bp.bp_profile_enable(False)
    bp.bp_profile_select(None)
    return med


def main():
    bp.load_library()
    dev = "cuda:0"
    n = 1 << 21                                          # rows fetched per launch
    print(f"{'row B':>6s} {'in flight':>9s} {'us':>8s} {'rows/us':>8s} {'GB/s rows':>10s} {'GB/s 128B lines':>16s}", flush=True)
    for rb in (64, 128, 192, 256, 384, 512):
        rows_total = (2 << 30) // rb                     # a 2 GiB table
        table = torch.empty((rows_total, rb // 4), dtype=torch.float32, device=dev).normal_()
        g = torch.Generator(device=dev).manual_seed(rb)
        lists = [torch.randint(0, rows_total, (n,), device=dev, generator=g, dtype=torch.int64).to(torch.int32)
                 for _ in range(4)]
        # 128-byte lines a row of rb bytes touches at an rb-byte stride, averaged over the alignments that occur
        offs = {(k * rb) % 128 for k in range(128)}
        lines = sum(math.ceil((o + rb) / 128) for o in offs) / len(offs)
        for u in (1, 2, 4, 8):
            sink = torch.empty((-(-n // u) + 256) * 4, dtype=torch.int32, device=dev)
            us = median_us(lambda k: bp.bp_gather_calibration(table, lists[k % 4], rows_in_flight=u, sink=sink))
            print(f"{rb:6d} {u:9d} {us:8.1f} {n / us:8.1f} {n * rb / us / 1e3:10.0f} {n * lines * 128 / us / 1e3:16.0f}",
                  flush=True)
        del table, lists
    print()
    print(f"{'row B':>6s} {'rows':>9s} {'order':>10s} {'in flight':>9s} {'us':>8s} {'rows/us':>8s} {'GB/s rows':>10s}", flush=True)
    for rb in (64, 128, 192, 256, 512):
        for rows_total in (425984, 1 << 21):             # one Criteo-shaped batch of one-lookup bags; 2 M rows
            tables = [torch.empty((rows_total, rb // 4), dtype=torch.int32, device=dev) for _ in range(4)]
            g = torch.Generator(device=dev).manual_seed(rb)
            orders = {"random": [torch.randperm(rows_total, device=dev, generator=g).to(torch.int32) for _ in range(4)],
                      "ascending": [torch.arange(rows_total, device=dev, dtype=torch.int32)] * 4}
            for name, lists in orders.items():
                for u in (1, 2, 4):
                    us = median_us(lambda k: bp.bp_scatter_calibration(tables[k % 4], lists[k % 4], rows_in_flight=u))
                    print(f"{rb:6d} {rows_total:9d} {name:>10s} {u:9d} {us:8.1f} {rows_total / us:8.1f} "
                          f"{rows_total * rb / us / 1e3:10.0f}", flush=True)
            del tables, orders


if __name__ == "__main__":
    main()
