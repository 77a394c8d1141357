"""CPU oracles for the MoE verification path — TEST INFRASTRUCTURE.

Only tests/, the smoke check and the bench's cpu_baseline leg may import this
package.  Nothing here imports, or is imported by, the HIP library or its binding.
"""
