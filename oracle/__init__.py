"""CPU oracle of the MoE-layer hot path.  TEST INFRASTRUCTURE ONLY: the product
package never imports this; tests, the smoke check and the benchmark's
cpu_baseline leg do."""
