"""CPU oracle -- TEST INFRASTRUCTURE ONLY (tests, smoke check, benchmark cpu_baseline leg).
The product package never imports this; this package never imports the product's HIP binding."""
