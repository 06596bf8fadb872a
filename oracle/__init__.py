"""CPU oracle: plain, slow reference implementations written from the paper and the textbook definitions.

TEST INFRASTRUCTURE ONLY.  Only tests, the smoke check and the benchmark's CPU-baseline leg may import this
package; the GPU library and its Python binding never do, and this package imports neither of them.
"""
