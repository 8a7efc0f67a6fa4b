"""TEST INFRASTRUCTURE ONLY: independent fp64 CPU oracle (see ssd_ref.py, magc_ref.py).

The product package never imports this; only tests, the smoke check and the
benchmark's cpu_baseline leg do."""
