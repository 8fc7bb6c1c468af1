"""MI355X-native VMoBA block-sparse attention hot path (arxiv 2506.23858).

The compute lives in the HIP library built from csrc/ (libvmoba.so, C ABI declared in
include/vmoba.h).  `paper_2506_23858_amd.binding` marshals arguments to it; `synth`
draws the seeded synthetic inputs.  Importing the package loads nothing.
"""
