"""Tolerances of the GPU parity tests (no imports: read by test modules at collection time).

Against the oracle in its default mode (which carries activations like the kernels do, as two bf16
terms): rel-L2 on logits and hidden states, and beside it the largest single deviation in units of the
oracle vector's rms, so that one wrong element cannot hide in the norm of 10^5 right ones.  The required
bars are 1e-5 (fp32 models) and 2e-2 (bf16 models); measured on the GPU: fp32 at most 8.4e-7 with a
largest deviation of 3.8e-6 rms; bf16 at most 2.2e-4 / 7.7e-4 rms on the paths the library takes by
itself (6.7e-4 / 3.2e-3 rms where the tests force matrix-core attention onto tiny models), and
2.7e-5 ... 9.3e-5 / 7.2e-4 rms at the full-size shapes, hence the tighter full-size figure.
Against the plain oracle (activations unrounded, RMSNorm as written, bf16 only in weights and cache):
the bar required of a bf16 model; measured at most 1.7e-4.
Token ids are compared wherever the oracle's top-1/top-2 gap exceeds MARGIN standard deviations of its
logits (a genuine near-tie cannot fail a correct kernel); the comparisons set aside are counted and
asserted few."""
TOL = {"fp32": 1e-5, "bf16": 1e-3}
FULL_SIZE_TOL = 3e-4          # bf16, the 8B / 7B shapes at full depth
PEAK_PER_TOL = 5.0            # largest single deviation allowed: PEAK_PER_TOL * tolerance, in units of rms(oracle vector)
MARGIN = {"fp32": 1e-5, "bf16": 1e-3}
PLAIN_TOL = 2e-2
