"""CPU oracle (test infrastructure only): a plain float64 statement of FP8 3D sliding-tile
attention written from the paper.  Imported only by tests, the smoke check and the benchmark's
cpu_baseline leg; the product package never imports it and shares no code with it."""
