"""CPU oracle of the RelServe layer step: test infrastructure only.

Only tests, the smoke check and the benchmark's cpu_baseline leg import this
package; the GPU library and its Python binding never do.
"""
