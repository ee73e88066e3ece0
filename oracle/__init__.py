"""CPU oracle for the FlatQuant online path (test infrastructure, not product code).

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
package.  It shares no code with the HIP library and never imports it.
"""
