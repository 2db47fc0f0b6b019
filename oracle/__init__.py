"""TEST INFRASTRUCTURE - slow, plain CPU reference of the reranker scoring pass.

Nothing here is part of the product path.  Only `tests/`, the smoke check and
the benchmark's CPU-baseline leg import it; it imports nothing from the GPU
package and shares no code with it.
"""
