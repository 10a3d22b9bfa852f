"""CPU oracle for the fused optimizer step + weight prediction.

Test infrastructure only: imported by ``tests/``, by ``__graft_entry__.smoke()``
and by the ``cpu_baseline`` leg of ``bench.py``.  Nothing in the GPU package
imports it and it imports nothing from the GPU package.
"""
from .po_oracle import (  # noqa: F401
    SGDM, ADAM, ADAMW, NESTEROV, RMSPROP, ADAGRAD, OracleLib, SOURCE, compile_source, build, step_predict, predict, bf16_from_f32, f32_from_bf16,
    version_difference,
)
