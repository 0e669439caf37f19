"""Roofs the benchmark's fractions are quoted against: MI355X's published peaks, and beside them the
rates measured on this machine with the library's own probe kernels (`bench.py --probe`; the run behind
the figures below is kept in profiles/roof_probes.md)."""

CUS = 256
CLOCK_HZ = 2.4e9

# published
HBM_PEAK = 8.0e12                              # B/s
LDS_PEAK = CUS * 256 * CLOCK_HZ                # 256 B/clk/CU for wide LDS reads: 157.3 TB/s
VALU_PEAK_FMA = CUS * 64 * CLOCK_HZ            # non-packed fp32 multiply-adds per second: 4 SIMDs x 16 lanes per CU
                                               # (78.6 TFLOP/s; the 157.3 TFLOP/s datasheet figure is the packed form,
                                               # which this build does not use)
VALU_PEAK_FMA_PACKED = 2 * VALU_PEAK_FMA

# measured with `bench.py --probe` (profiles/roof_probes.md)
MEASURED_LDS_B_PER_CLK_PER_CU = 229.4          # ds_read_b128, 64 consecutive elements per wavefront, 16 wavefronts per CU
MEASURED_COPY_BYTES_PER_S = 4.62e12            # read + write bytes of a 1 GiB copy
PROFILE = "profiles/roof_probes.md"

# HBM-side bytes per launch of sc::tile_kernel (scaled FETCH_SIZE + WRITE_SIZE, mean over the launches of a step),
# from the rocprofv3 --pmc runs kept under profiles/ (each names the commit it was taken at).  A bench run does
# not count bytes; it reports these for the workloads they were measured on, in their default configuration.
MEASURED_TRAFFIC_BYTES_PER_LAUNCH = {
    "vgg16_f32": (35.9e6, "profiles/tile_kernel_vgg16_f32_n128_hbm_traffic.md"),
    "vgg16_f16": (40.5e6, "profiles/tile_kernel_vgg16_f16_n256_hbm_traffic.md"),
}
