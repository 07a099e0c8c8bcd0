"""CPU oracle (test infrastructure only): see quasar_ref.py and quasar_ref.c.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
package.  It shares no code with the HIP library or its Python binding.
"""
