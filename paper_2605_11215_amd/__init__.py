"""MI355X-native implementation of the ReCoVer data-parallel gradient path.

`binding` wraps the C-ABI library (include/recover.h) one to one; `synth` makes the seeded
synthetic inputs.  Importing this package loads nothing; `binding.lib()` loads the built
shared library and raises if it is missing (there is no CPU path).
"""
