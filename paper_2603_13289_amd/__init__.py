"""MI355X-native selective-recompute prefill (RelayCaching): HIP kernels behind a C ABI.

`paper_2603_13289_amd.binding` loads librelaycache.so and mirrors its entry
points; importing it fails if the library has not been built
(`python -m paper_2603_13289_amd.build`).  It is not imported here so that the
build module itself can be run before the library exists.
"""
