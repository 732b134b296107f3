"""MI355X-native hot path of distributed auto-differentiation (dAD).

The arithmetic lives in the HIP library (csrc/, built to libdad.so); `binding`
only marshals arguments across its C ABI.  `workloads` draws synthetic inputs.
"""
