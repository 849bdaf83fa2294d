"""MI355X-native weight-only-quantized fully-connected layer (decode GEMV,
prefill GEMM) behind a C-ABI library.  Import ``paper_2505_00232_amd.binding``
for the GPU path and ``paper_2505_00232_amd.synth`` for the seeded workloads;
this file imports neither, so the input generators can be used without the
compiled library."""
