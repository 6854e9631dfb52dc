"""TEST INFRASTRUCTURE -- the CPU oracle of the sharded optimizer step.

Only ``tests/``, the smoke check and the benchmark's CPU-baseline leg may
import this package.  It holds a plain definition of what the step computes
(``step.c`` behind ``oracle.step``) and of the placement closed forms
(``oracle.placement``).  Nothing here touches a GPU, and the GPU library
neither imports nor links any of it.
"""
