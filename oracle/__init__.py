"""CPU oracle for the KV-Runahead chunked-prefill hot path (test infrastructure only).

Nothing under this package is part of the product path: it may be imported only by the
test-suite, by the repository's smoke check and by the benchmark's cpu_baseline leg.
It shares no code with the HIP library and never imports it.
"""
