"""CPU oracle for Hybrid Target Attention.  Test infrastructure only: nothing in the product
package may import this; only tests/, the smoke check and the benchmark's cpu_baseline leg do."""
