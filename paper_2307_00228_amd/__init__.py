"""MI355X-native hot path of full-graph GNN inference in the Gather-Apply-Scatter schema.

``workloads`` draws seeded synthetic inputs; ``binding`` marshals arguments for the
C-ABI HIP library (``libinferturbo_hip.so``, built by ``build.build()``).  Nothing
here falls back to the CPU: without the built library the binding raises.
"""
