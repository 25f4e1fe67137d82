"""TEST INFRASTRUCTURE: the CPU oracle for batched critical-path evaluation.

Only tests, the smoke check and the benchmark's CPU-baseline leg import this
package.  It never imports the GPU package, and the GPU package never imports it.
"""
