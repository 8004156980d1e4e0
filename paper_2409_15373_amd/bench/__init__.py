"""Measurement programs around the library (run as `python -m paper_2409_15373_amd.bench.<name>`): timings of all
configurations, the comparisons of Section 3 / Figure 2 and Table 1, and the variants.  Nothing here is on the
product path; every module only calls the C ABI through `binding`."""
