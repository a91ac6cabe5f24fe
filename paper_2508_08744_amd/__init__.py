"""MI355X-native GNN-Descent k-NN graph construction (hand-written HIP behind a C-ABI).

``paper_2508_08744_amd.knn`` is the Python binding of the C-ABI library;
``paper_2508_08744_amd.inputs`` holds the seeded synthetic input generators.
The binding is imported lazily so that the generators can be used without the
HIP library being present.
"""

__all__ = ["inputs", "knn"]
