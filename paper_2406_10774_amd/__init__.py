"""Quest decode hot path (arXiv 2406.10774) for AMD MI355X: HIP kernels behind a
C ABI (include/quest.h) plus this thin ctypes binding.

    from paper_2406_10774_amd import binding as quest
    quest.quest_build_meta(cache) ...

`synth` holds the seeded synthetic workloads used by tests and the benchmark."""
