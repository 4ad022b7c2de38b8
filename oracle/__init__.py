"""Test infrastructure only: the fp64 brute-force oracle for knowledge-base retrieval.

Only the tests, the smoke check and the benchmark's cpu_baseline leg may import this
package; the product path never does.
"""
