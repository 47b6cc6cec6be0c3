"""CPU oracle for one CoCoD-SGD round (Algorithm 1) -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
package.  It shares no code with the HIP library and never imports it.
"""
