"""Collage MCF-AdamW optimizer step for MI355X (gfx950): C-ABI library plus a thin ctypes binding.

    from paper_2405_03637_amd import binding as mcf      # mcf.Plan, mcf.adamw_step_flat, mcf.fast2sum, ...
    from paper_2405_03637_amd import workloads           # seeded synthetic parameter sets
    from paper_2405_03637_amd import build               # build.build() compiles libmcf_adamw.so with hipcc

Nothing is imported eagerly: loading the library needs torch (for its HIP runtime) and a built .so.
"""
