"""CPU oracle for the TailorKV decode-attention hot path (arxiv 2505.19586).

TEST INFRASTRUCTURE ONLY.  Plain, slow numpy in float64 (float32 where a step
decides an integer or a stored fp16 value, see each function).  Nothing under
the product package imports this; only tests, the smoke check and the
benchmark's cpu_baseline leg call it.  It shares no code, tables or helpers
with the HIP path.

Parity status of each function against the paper:
  * quantizer (Sec. 2.2, Eq. 4), attention (Sec. 2.1, Eq. 3) and the memory
    model (Sec. 4.4, Table 2) are pinned by closed forms, invariants and
    brute force in tests/test_oracle_*.py;
  * the dense preference score (Sec. 4.1, Eq. 6-9) is pinned by closed forms
    (uniform and one-hot attention), brute force and monotonicity in
    tests/test_oracle_preference.py;
  * the paper prints no worked numeric example for this path, so beyond the
    Table 2 closed form there is no paper-printed value to compare with.
"""
from . import attention, layout, preference, quant, sparse  # noqa: F401
