"""TEST INFRASTRUCTURE ONLY.

Slow, plain CPU oracle for the predict / verify / commit decode path of an
hourglass transformer over mesh coordinate tokens.  Imported only by tests, the
smoke check and the benchmark's cpu_baseline leg; shares no code with the HIP
path.
"""
