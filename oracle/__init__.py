"""CPU oracle: TEST INFRASTRUCTURE ONLY.

Plain, slow definitions of what the HIP path must compute (operators in `ops`,
the schedule-construction walk in `construct`).  Nothing here is imported by the
product package; only tests, the smoke check and the benchmark's cpu_baseline leg use it.
"""
