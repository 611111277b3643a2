"""MI355X-native conv1d sub-block (forward, input gradient, weight gradient) of the
Jasper-style acoustic encoder.  The compute lives in the HIP library under ``csrc/``;
``binding`` marshals arguments to its C ABI and ``inputs`` draws the synthetic workloads.
Importing the package loads nothing heavy; ``binding.lib()`` loads the HIP library and
raises if it has not been built."""

__all__ = ["binding", "inputs"]
