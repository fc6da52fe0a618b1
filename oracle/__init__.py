"""CPU oracle of the TAH-Quant activation codec.  TEST INFRASTRUCTURE ONLY.

Nothing in the product path may import this package: it is loaded by the tests,
by the smoke check and by the cpu_baseline leg of the benchmark, and it imports
nothing from the HIP library or its Python binding.

  o32  -- the plain-C oracle (fp32 operation order), through ctypes
  o64  -- a float64 NumPy transcription of the paper's equations, used to pin o32
"""
