"""MI355X-native node-centric equivariant attention forward (E2Former-V2 hot path).

The compute lives in the HIP library built from csrc/ and is reached through `binding`; `workloads`
holds the seeded synthetic inputs.  Importing this package does not load the HIP library.
"""
