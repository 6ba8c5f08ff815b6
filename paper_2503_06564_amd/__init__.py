"""MI355X-native rotated W8A8 / W4A8 linear of TR-DQ (hand-written HIP behind a C ABI).

`paper_2503_06564_amd.trdq` is the ctypes binding of libtrdq.so;
`paper_2503_06564_amd.workloads` the seeded synthetic inputs.  Importing the
package loads nothing; the binding raises if the HIP library has not been built.
"""
