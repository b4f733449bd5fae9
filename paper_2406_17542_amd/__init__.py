"""CDQuant hot path for AMD MI355X (gfx950): Hessian, grid/RTN init, greedy coordinate
descent and loss, as hand-written HIP behind a C ABI (``include/cdq.h``).

``paper_2406_17542_amd.cdq`` is the thin binding over ``libcdq.so``;
``paper_2406_17542_amd.inputs`` holds the seeded synthetic-layer recipes."""
