"""MI355X-native transformer-layer forward/backward with activation offloading.

The compute lives in the HIP shared library under `csrc/`; `binding` marshals arguments
to its C ABI and `synth` generates the seeded synthetic workloads.  Importing the package
loads nothing: the library is opened on first use and its absence is an error.
"""
