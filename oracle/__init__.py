"""fp64 CPU oracle for the batched block-compaction layer.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this
package; it exists so that tests, the smoke check and the CPU-baseline leg of
the benchmark can compare the HIP kernels against a plain definition.
"""
