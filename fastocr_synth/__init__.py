"""Seeded synthetic inputs for the FastOCR decode hot path.

Input generation only: counter-based random numbers, cache layouts and the
drifting-fixation query process.  None of the method's arithmetic (no logits,
softmax, selection or attention) lives here, so both the CPU oracle's tests and
the HIP path's tests/benchmark may draw their inputs from this one module.

Everything is a pure function of (seed, coordinates): any element of any tensor
can be regenerated without generating the rest.  Tensors are torch tensors on
the requested device (CPU here, the GPU in the benchmark); a bf16 cache is
handed to the oracle as its raw uint16 bit pattern via ``to_oracle_array``.

Stand-in for the documents of the paper's OCR benchmarks pushed through a
Qwen2.5-VL-class model: K, V ~ N(0,1) for every cached token; the query of a
step is the mean key of a small window of the visual grid (the "fixation") plus
N(0, sigma^2) noise, and the window centre drifts in raster order by one or two
cells per step -- the gradual shift of fixation the paper observes.
"""
from .rng import normal_rows, uniform_u64  # noqa: F401
from .workloads import (  # noqa: F401
    BASE_SEED,
    Workload,
    Batch,
    config,
    make_batch,
    centres,
    queries_for_step,
    to_oracle_array,
    window_cells,
)
