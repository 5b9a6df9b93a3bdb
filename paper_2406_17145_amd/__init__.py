"""MI355X-native graph-pipeline-parallel stage: C-ABI HIP library + thin binding.

Importing the package does not load the native library; `binding.load()` does,
and fails loudly when the library has not been built.
"""
