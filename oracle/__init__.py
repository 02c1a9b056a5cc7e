"""CPU oracle for the conv2d path.  TEST INFRASTRUCTURE ONLY: imported by
tests/, by the smoke check and by the bench's cpu_baseline leg; never by the
product package."""
