"""Seeded synthetic inputs shared by the tests, the smoke check and the
benchmark.  Holds none of the method's arithmetic (no LayerNorm, projection,
softmax, exit rule or verification) and imports neither the oracle nor the HIP
binding."""
