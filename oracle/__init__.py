"""CPU oracle for the COMP-AMS step: test infrastructure only.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
package; the GPU library never does.
"""
