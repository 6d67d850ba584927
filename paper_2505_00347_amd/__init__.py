"""SOLO low-bit AdamW step for AMD MI355X: HIP kernels behind a C-ABI library.

``paper_2505_00347_amd.solo`` is the binding of ``include/solo.h``;
``paper_2505_00347_amd.synth`` holds the seeded synthetic workloads;
``paper_2505_00347_amd.build`` compiles the library with hipcc.
"""
