"""CPU oracle of the F8Net fixed-point layer arithmetic: test infrastructure only.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
package.  It shares no code with the GPU library.
"""
