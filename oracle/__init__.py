"""CPU oracle (test infrastructure only): the slow, plain definition of every step.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
package.  It shares nothing with the HIP library.
"""
