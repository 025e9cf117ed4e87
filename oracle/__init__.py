"""CPU checker (test infrastructure only).

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
package; the product path never does.
"""
