"""MI355X-native hot path of DepCap block-wise diffusion-LM decoding.

The compute lives in the C-ABI library built from csrc/ (see include/dlm.h);
`api` is the thin ctypes binding with the same entry-point names, `decode` the
host loop that strings the entry points into a full block-wise decode, and
`inputs` the seeded synthetic workloads.  Importing the package loads nothing
native; the library is opened on first use and its absence is an error.
"""
