"""CPU oracle for the Pro-GRPO pruned-sampling path.

TEST INFRASTRUCTURE ONLY.  Everything under this package is a plain, slow,
fp64 NumPy restatement of what the sampling loop of the paper computes
(Sec. 3, Sec. 4.2, Sec. 5.1, Sec. 5.2).  It exists so that the HIP library can
be checked element by element.  Only the tests, the smoke entry and the
``cpu_baseline`` leg of the benchmark may import it; the product package never
does, and nothing in here imports the product package.

Pins (what ties each routine to something other than itself) are listed in the
header of each module; the tests under ``tests/`` marked "not gpu" execute them.
"""
